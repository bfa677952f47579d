// Internal declarations shared by the translation units of libkvcapsule.so.
// Nothing here is part of the C ABI (include/kvcapsule.h is).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/kvcapsule.h"
#include "../../include/kvcapsule_dev.h"

namespace kvc {

// ---- element types -------------------------------------------------------------
struct bf16_t {
    uint16_t v;
};

__host__ __device__ inline float to_f(float x) { return x; }
__device__ inline float to_f(bf16_t x) { return __uint_as_float(static_cast<uint32_t>(x.v) << 16); }

// round-to-nearest-even fp32 -> bf16 bits: gfx950 converts in hardware (one packed instruction
// per pair of values)
__device__ inline uint16_t f32_to_bf16_bits(float f)
{
    return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));
}

template <class T> __device__ inline T from_f(float f);
template <> __device__ inline float from_f<float>(float f) { return f; }
template <> __device__ inline bf16_t from_f<bf16_t>(float f) { return bf16_t{f32_to_bf16_bits(f)}; }

// ---- layout of the compressed values of one image block --------------------------------
// The m rows are grouped in blocks of 8; a block holds [d][w] with w = 8 (w = m % 8 for a
// last, shorter block), i.e. 8 consecutive rows of one channel are 16 contiguous bytes in
// bf16: exactly the operand a 16x16x32 MFMA lane needs for out = W Vc.  No padding: the
// record has m*d elements.  Offset of (row j, channel c):
__host__ __device__ inline size_t vc_offset(int j, int c, int m, int d)
{
    const int jb = j >> 3;
    const int w = (m - 8 * jb) < 8 ? (m - 8 * jb) : 8;
    return static_cast<size_t>(jb) * 8 * d + static_cast<size_t>(c) * w + (j & 7);
}

// ---- wavefront (64 lanes) reductions --------------------------------------------
__device__ inline float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}
__device__ inline float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}

// ---- one decode call, validated ----------------------------------------------------
struct DecodeCall {
    kvc_shape s;
    const void *theta, *U, *mu;
    const void *theta_packed = nullptr;   // theta in the blocked form of kvc_pack_theta, or null
    const void *U_packed = nullptr;       // U in the blocked form of kvc_pack_u, or null
    const void *q, *Kc, *Vc;
    void *Kt, *Vt;
    int32_t t;        // text rows attended (new token included when appended)
    int32_t t_in;     // rows valid before the call; the new token goes to this row
    int32_t cap;
    const void *k_new, *v_new;
    float scale;
    void *out;
    float *lse;
    void *ws;
    size_t ws_bytes;
    hipStream_t stream;
    // ragged call (scalar kernels): per-sequence image-block and text-row counts in device memory, or null;
    // t and t_in then hold the largest values any sequence may have
    const int32_t *n_images_dev = nullptr, *text_len_dev = nullptr;
    bool static_variant = false;      // attend the compressed rows themselves (no theta, U, mu)
};

struct CompressCall {
    kvc_shape s;
    const int32_t *key_idx;
    const void *U, *mu;
    const void *K, *V;
    int64_t stride_b, stride_h, stride_s;
    int32_t vis_start;
    void *Kc, *Vc;
    void *ws;
    size_t ws_bytes;
    hipStream_t stream;
};

// full-cache decode attention (the "All KV" comparison point), validated
struct FullCall {
    int B, Hq, Hkv;
    const void *q;
    void *K, *V;
    long sb, sh, ss;  // element strides of the cache [B][H_kv][cap][d]
    int32_t t;        // rows attended (new token included when appended)
    int32_t t_in;     // rows valid before the call; the new token goes to this row
    const void *k_new, *v_new;
    float scale;
    void *out;
    float *lse;
    void *ws;
    size_t ws_bytes;
    hipStream_t stream;
    int cus;          // compute units of the device (0: ask the runtime)
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Raises a kernel's dynamic-LDS limit once per device (the attribute is per device); `done` is the
// caller's static flag array for that kernel.  False: the launch must not go ahead.
constexpr int kMaxDevices = 64;
inline bool allow_lds(const void *fn, size_t bytes, bool *done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
    if (done[dev]) return true;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes)) != hipSuccess) return false;
    done[dev] = true;
    return true;
}

// scalar (shape-agnostic) path
size_t generic_decode_ws_bytes(const kvc_shape &s, int32_t max_text);
kvc_status generic_decode(const DecodeCall &c);
kvc_status generic_compress(const CompressCall &c);
kvc_status generic_mlp_hidden(const kvc_shape &s, const void *W1, int act, const void *Kc, void *H, hipStream_t stream);

// matrix-core path for bf16, head_dim 128
bool fast_decode_supported(const kvc_shape &s);
size_t fast_decode_ws_bytes(const kvc_shape &s, int32_t max_text);
kvc_status fast_decode(const DecodeCall &c);
void fast_decode_knobs(int row_tiles, int separate, int wait_ticks);
long fast_decode_fallbacks();
// merges nparts part records ([G][128] un-normalised outputs, [G] maxima, [G] sums; the first nvp
// of them vision parts, whose probability mass multiplies mu) of every (batch element, query
// head) into out / lse; nparts <= 64
kvc_status finalize_parts(const float *Ypart, int nparts, int nvp, int rec, int B, int Hq, int Hkv, const void *mu,
                          void *out, float *lse, hipStream_t stream);
// shared by the decode paths that synchronise workgroups through counters in the workspace
unsigned next_decode_epoch();
int decode_wait_ticks();
unsigned *decode_fallback_counter();
// one-pass ("stream") decode for bf16, head_dim 128, theta in packed form: true when the call was taken
bool stream_decode(const DecodeCall &c, kvc_status *st);
size_t stream_decode_ws_bytes(const kvc_shape &s, int32_t max_text);
void stream_decode_knob(int mode);
long stream_decode_calls();
kvc_status pack_theta(const kvc_shape &s, const void *theta, void *packed, hipStream_t stream);
kvc_status pack_u(const kvc_shape &s, const void *U, void *packed, hipStream_t stream);
// full-cache decode, bf16, head_dim 128
bool fast_full_supported(int dtype, int head_dim, int G);
size_t fast_full_ws_bytes(int B, int Hq, int Hkv);
kvc_status fast_full_decode(const FullCall &c);
void full_decode_set_chunk_steps(int steps);
bool fast_compress_supported(const kvc_shape &s);
size_t fast_compress_ws_bytes(const kvc_shape &s);
kvc_status fast_compress(const CompressCall &c);
void fast_compress_knobs(int waves, int jt);

}  // namespace kvc
