// C ABI of libkvcapsule.so: argument validation, host-side closed forms and dispatch.
// Every check happens before the first HIP call, so a negative status means that
// nothing touched the device.
#include <math.h>

#include <algorithm>
#include <mutex>

#include "kvc_internal.h"

using namespace kvc;

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

kvc_status check_shape(const kvc_shape *s)
{
    if (!s) return KVC_ERR_NULL;
    if (s->dtype != KVC_F32 && s->dtype != KVC_BF16) return KVC_ERR_DTYPE;
    if (s->batch < 1 || s->n_kv_heads < 1 || s->n_q_heads < 1) return KVC_ERR_SHAPE;
    if (s->n_q_heads % s->n_kv_heads != 0) return KVC_ERR_SHAPE;
    if (s->head_dim < 8 || s->head_dim % 8 != 0) return KVC_ERR_SHAPE;
    if (s->n_img_tokens < 1 || s->n_images < 0) return KVC_ERR_SHAPE;
    if (s->m < 1 || s->m > s->n_img_tokens) return KVC_ERR_SHAPE;
    if (s->head_dim > 256) return KVC_ERR_UNSUPPORTED;
    // launch-grid limits of the kernels (grid.y / grid.z carry these products)
    if (static_cast<int64_t>(s->batch) * s->n_q_heads > 65535) return KVC_ERR_UNSUPPORTED;
    if (s->n_images > 65535) return KVC_ERR_UNSUPPORTED;
    // 32-bit row counters inside the kernels
    if (static_cast<int64_t>(s->n_images) * s->n_img_tokens > (1 << 30)) return KVC_ERR_UNSUPPORTED;
    return KVC_OK;
}

kvc_status check_params(const kvc_params *p, bool need_idx, bool need_theta)
{
    if (!p) return KVC_ERR_NULL;
    if (!p->U || !p->mu) return KVC_ERR_NULL;
    if (need_idx && !p->key_idx) return KVC_ERR_NULL;
    if (need_theta && !p->theta) return KVC_ERR_NULL;
    if (!aligned16(p->U) || !aligned16(p->mu)) return KVC_ERR_ALIGN;
    if (need_theta && (!aligned16(p->theta) || !aligned16(p->theta_packed) || !aligned16(p->U_packed))) return KVC_ERR_ALIGN;
    if (need_idx && (reinterpret_cast<uintptr_t>(p->key_idx) & 3u)) return KVC_ERR_ALIGN;
    return KVC_OK;
}

kvc_status prepare_decode(DecodeCall &c, const kvc_shape *shape, const kvc_params *params,
                          const void *q, const void *Kc, const void *Vc, void *K_text,
                          void *V_text, int32_t text_len, int32_t text_cap, const void *k_new,
                          const void *v_new, float softmax_scale, void *out, float *lse_out,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    kvc_status st = check_shape(shape);
    if (st != KVC_OK) return st;
    st = check_params(params, false, true);
    if (st != KVC_OK) return st;
    if (!q || !out) return KVC_ERR_NULL;
    if (shape->n_images > 0 && (!Kc || !Vc)) return KVC_ERR_NULL;
    if (text_cap < 0 || text_len < 0 || text_len > text_cap) return KVC_ERR_SHAPE;
    if ((k_new == nullptr) != (v_new == nullptr)) return KVC_ERR_NULL;
    if (k_new && text_len + 1 > text_cap) return KVC_ERR_SHAPE;
    if (text_cap > 0 && (!K_text || !V_text)) return KVC_ERR_NULL;
    const int32_t t = text_len + (k_new ? 1 : 0);
    if (shape->n_images == 0 && t == 0) return KVC_ERR_SHAPE;   // softmax over no key
    if (!(softmax_scale >= 0.f) || isinf(softmax_scale)) return KVC_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(out) || !aligned16(Kc) || !aligned16(Vc) ||
        !aligned16(K_text) || !aligned16(V_text) || !aligned16(k_new) || !aligned16(v_new) ||
        (reinterpret_cast<uintptr_t>(lse_out) & 3u))
        return KVC_ERR_ALIGN;
    if (!workspace) return KVC_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return KVC_ERR_ALIGN;
    c.s = *shape;
    c.theta = params->theta;
    c.theta_packed = params->theta_packed;
    c.U_packed = params->U_packed;
    c.U = params->U;
    c.mu = params->mu;
    c.q = q;
    c.Kc = Kc;
    c.Vc = Vc;
    c.Kt = K_text;
    c.Vt = V_text;
    c.t = t;
    c.t_in = text_len;
    c.cap = text_cap;
    c.k_new = k_new;
    c.v_new = v_new;
    c.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf(static_cast<float>(shape->head_dim));
    c.out = out;
    c.lse = lse_out;
    c.ws = workspace;
    c.ws_bytes = workspace_bytes;
    c.stream = static_cast<hipStream_t>(stream);
    return KVC_OK;
}

kvc_status prepare_compress(CompressCall &c, const kvc_shape *shape, const kvc_params *params,
                            const void *K, const void *V, int64_t stride_b, int64_t stride_h,
                            int64_t stride_s, int32_t vis_start, int32_t seq_len, void *Kc, void *Vc,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    kvc_status st = check_shape(shape);
    if (st != KVC_OK) return st;
    st = check_params(params, true, false);
    if (st != KVC_OK) return st;
    if (shape->n_images > 0 && (!K || !V || !Kc || !Vc)) return KVC_ERR_NULL;
    if (vis_start < 0 || seq_len < 0) return KVC_ERR_SHAPE;
    // the vision span lies inside the sequence
    if (static_cast<int64_t>(vis_start) + static_cast<int64_t>(shape->n_images) * shape->n_img_tokens > seq_len)
        return KVC_ERR_SHAPE;
    if (stride_s < shape->head_dim || stride_h < 0 || stride_b < 0) return KVC_ERR_SHAPE;
    if (stride_s % 8 || stride_h % 8 || stride_b % 8) return KVC_ERR_ALIGN;
    if (!aligned16(K) || !aligned16(V) || !aligned16(Kc) || !aligned16(Vc)) return KVC_ERR_ALIGN;
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return KVC_ERR_ALIGN;
    c.s = *shape;
    c.key_idx = params->key_idx;
    c.U = params->U;
    c.mu = params->mu;
    c.K = K;
    c.V = V;
    c.stride_b = stride_b;
    c.stride_h = stride_h;
    c.stride_s = stride_s;
    c.vis_start = vis_start;
    c.Kc = Kc;
    c.Vc = Vc;
    c.ws = workspace;
    c.ws_bytes = workspace_bytes;
    c.stream = static_cast<hipStream_t>(stream);
    return KVC_OK;
}

// the matrix-core kernels where the shape allows it, else the scalar kernels
kvc_status dispatch_decode(const DecodeCall &c)
{
    kvc_status st = KVC_OK;
    if (stream_decode(c, &st)) return st;
    if (fast_decode_supported(c.s)) return fast_decode(c);
    return generic_decode(c);
}

template <class T>
__global__ __launch_bounds__(256) void unpack_values(const T *__restrict__ Vc, T *__restrict__ dense, int m, int d)
{
    const T *src = Vc + static_cast<size_t>(blockIdx.x) * m * d;
    T *dst = dense + static_cast<size_t>(blockIdx.x) * m * d;
    for (int x = threadIdx.x; x < m * d; x += 256) {
        const int j = x / d, c = x - j * d;
        dst[x] = src[vc_offset(j, c, m, d)];
    }
}

}  // namespace

extern "C" {

int32_t kvc_compressed_len(int32_t n, double compression_ratio)
{
    if (n <= 0) return 0;
    // ceil((1 - c) n); the small backoff keeps exact-integer products such as
    // 0.5 * 576 from rounding up because (1 - c) is not exact in binary
    double v = ceil((1.0 - compression_ratio) * static_cast<double>(n) - 1e-9);
    if (!(v >= 1.0)) v = 1.0;
    if (v > static_cast<double>(n)) v = static_cast<double>(n);
    return static_cast<int32_t>(v);
}

size_t kvc_workspace_bytes(const kvc_shape *shape, int32_t max_text_len)
{
    if (check_shape(shape) != KVC_OK || max_text_len < 0) return 0;
    size_t need = generic_decode_ws_bytes(*shape, max_text_len);
    if (fast_decode_supported(*shape)) {
        size_t f = fast_decode_ws_bytes(*shape, max_text_len);
        if (f > need) need = f;
    }
    if (fast_compress_supported(*shape)) {
        size_t f = fast_compress_ws_bytes(*shape);
        if (f > need) need = f;
    }
    need = std::max(need, stream_decode_ws_bytes(*shape, max_text_len));
    return need;
}

kvc_status kvc_memory_footprint(const kvc_shape *shape, int64_t c_prompt, int64_t t,
                                int64_t *bytes_full_cache, int64_t *bytes_capsule)
{
    kvc_status st = check_shape(shape);
    if (st != KVC_OK) return st;
    if (c_prompt < 0 || t < 0) return KVC_ERR_SHAPE;
    const int64_t b = shape->dtype == KVC_F32 ? 4 : 2;
    const int64_t B = shape->batch, H = shape->n_kv_heads, d = shape->head_dim;
    const int64_t n = shape->n_img_tokens, I = shape->n_images, m = shape->m;
    if (bytes_full_cache) *bytes_full_cache = 2 * B * H * (c_prompt + I * n + t) * d * b;
    if (bytes_capsule)
        *bytes_capsule = 2 * B * H * (c_prompt + I * m + t) * d * b   // compressed KV cache
                         + H * m * n * b                               // theta
                         + H * m * n * b + H * d * b;                  // U and mu
    return KVC_OK;
}

kvc_status kvc_compress(const kvc_shape *shape, const kvc_params *params, const void *K,
                        const void *V, int64_t stride_b, int64_t stride_h, int64_t stride_s,
                        int32_t vis_start, int32_t seq_len, void *Kc, void *Vc, void *workspace,
                        size_t workspace_bytes, void *stream)
{
    CompressCall c;
    kvc_status st = prepare_compress(c, shape, params, K, V, stride_b, stride_h, stride_s,
                                     vis_start, seq_len, Kc, Vc, workspace, workspace_bytes, stream);
    if (st != KVC_OK) return st;
    if (fast_compress_supported(c.s)) return fast_compress(c);
    return generic_compress(c);
}

kvc_status kvc_compress_generic(const kvc_shape *shape, const kvc_params *params, const void *K,
                                const void *V, int64_t stride_b, int64_t stride_h,
                                int64_t stride_s, int32_t vis_start, int32_t seq_len, void *Kc, void *Vc,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    CompressCall c;
    kvc_status st = prepare_compress(c, shape, params, K, V, stride_b, stride_h, stride_s,
                                     vis_start, seq_len, Kc, Vc, workspace, workspace_bytes, stream);
    if (st != KVC_OK) return st;
    return generic_compress(c);
}

kvc_status kvc_reconstruct_attend_decode(const kvc_shape *shape, const kvc_params *params,
                                         const void *q, const void *Kc, const void *Vc,
                                         void *K_text, void *V_text, int32_t text_len,
                                         int32_t text_cap, const void *k_new, const void *v_new,
                                         float softmax_scale, void *out, float *lse_out,
                                         void *workspace, size_t workspace_bytes, void *stream)
{
    DecodeCall c;
    kvc_status st = prepare_decode(c, shape, params, q, Kc, Vc, K_text, V_text, text_len, text_cap,
                                   k_new, v_new, softmax_scale, out, lse_out, workspace,
                                   workspace_bytes, stream);
    if (st != KVC_OK) return st;
    return dispatch_decode(c);
}

kvc_status kvc_reconstruct_attend_decode_generic(const kvc_shape *shape, const kvc_params *params,
                                                 const void *q, const void *Kc, const void *Vc,
                                                 void *K_text, void *V_text, int32_t text_len,
                                                 int32_t text_cap, const void *k_new,
                                                 const void *v_new, float softmax_scale, void *out,
                                                 float *lse_out, void *workspace,
                                                 size_t workspace_bytes, void *stream)
{
    DecodeCall c;
    kvc_status st = prepare_decode(c, shape, params, q, Kc, Vc, K_text, V_text, text_len, text_cap,
                                   k_new, v_new, softmax_scale, out, lse_out, workspace,
                                   workspace_bytes, stream);
    if (st != KVC_OK) return st;
    return generic_decode(c);
}

// ---- variants that run on the shape-agnostic kernels -------------------------------------------------
kvc_status kvc_reconstruct_attend_decode_ragged(const kvc_shape *shape, const kvc_params *params,
                                                const void *q, const void *Kc, const void *Vc,
                                                void *K_text, void *V_text, const int32_t *n_images,
                                                const int32_t *text_len, int32_t text_cap,
                                                const void *k_new, const void *v_new, float softmax_scale,
                                                void *out, float *lse_out, void *workspace,
                                                size_t workspace_bytes, void *stream)
{
    if (!n_images || !text_len) return KVC_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(n_images) & 3u) || (reinterpret_cast<uintptr_t>(text_len) & 3u)) return KVC_ERR_ALIGN;
    if (text_cap < 1) return KVC_ERR_SHAPE;
    // validated as the uniform call with the longest text that fits
    const int32_t t_max = text_cap - (k_new ? 1 : 0);
    DecodeCall c;
    kvc_status st = prepare_decode(c, shape, params, q, Kc, Vc, K_text, V_text, t_max, text_cap, k_new, v_new,
                                   softmax_scale, out, lse_out, workspace, workspace_bytes, stream);
    if (st != KVC_OK) return st;
    c.n_images_dev = n_images;
    c.text_len_dev = text_len;
    return dispatch_decode(c);
}

kvc_status kvc_static_attend_decode(const kvc_shape *shape, const void *q, const void *Kc, const void *Vc,
                                    void *K_text, void *V_text, int32_t text_len, int32_t text_cap,
                                    const void *k_new, const void *v_new, float softmax_scale, void *out,
                                    float *lse_out, void *workspace, size_t workspace_bytes, void *stream)
{
    // theta, U and mu are not part of this variant; q stands in for them (never read)
    kvc_params none;
    none.key_idx = nullptr; none.theta = q; none.U = q; none.mu = q; none.theta_packed = nullptr; none.U_packed = nullptr;
    DecodeCall c;
    kvc_status st = prepare_decode(c, shape, &none, q, Kc, Vc, K_text, V_text, text_len, text_cap, k_new, v_new,
                                   softmax_scale, out, lse_out, workspace, workspace_bytes, stream);
    if (st != KVC_OK) return st;
    c.static_variant = true;
    return generic_decode(c);
}

kvc_status kvc_mlp_hidden(const kvc_shape *shape, const void *W1, int32_t activation, const void *Kc, void *H,
                          void *stream)
{
    kvc_status st = check_shape(shape);
    if (st != KVC_OK) return st;
    if (activation < KVC_ACT_IDENTITY || activation > KVC_ACT_GELU) return KVC_ERR_SHAPE;
    if (!W1) return KVC_ERR_NULL;
    if (shape->n_images > 0 && (!Kc || !H)) return KVC_ERR_NULL;
    if (Kc == H) return KVC_ERR_SHAPE;                       // every output row reads all input rows
    if (!aligned16(W1) || !aligned16(Kc) || !aligned16(H)) return KVC_ERR_ALIGN;
    return generic_mlp_hidden(*shape, W1, activation, Kc, H, static_cast<hipStream_t>(stream));
}

kvc_status kvc_pack_theta(const kvc_shape *shape, const void *theta, void *packed, void *stream)
{
    kvc_status st = check_shape(shape);
    if (st != KVC_OK) return st;
    if (!theta || !packed) return KVC_ERR_NULL;
    if (theta == packed) return KVC_ERR_SHAPE;
    if (!aligned16(theta) || !aligned16(packed)) return KVC_ERR_ALIGN;
    return pack_theta(*shape, theta, packed, static_cast<hipStream_t>(stream));
}

kvc_status kvc_pack_u(const kvc_shape *shape, const void *U, void *packed, void *stream)
{
    kvc_status st = check_shape(shape);
    if (st != KVC_OK) return st;
    if (!U || !packed) return KVC_ERR_NULL;
    if (U == packed) return KVC_ERR_SHAPE;
    if (!aligned16(U) || !aligned16(packed)) return KVC_ERR_ALIGN;
    if (shape->n_img_tokens % 8) return KVC_ERR_UNSUPPORTED;         // whole blocks of 8 positions
    return pack_u(*shape, U, packed, static_cast<hipStream_t>(stream));
}

// ---- the blocked layout of the compressed values, for callers ---------------------------------------
int64_t kvc_capsule_value_offset(int32_t j, int32_t c, int32_t m, int32_t d)
{
    if (m < 1 || d < 1 || j < 0 || j >= m || c < 0 || c >= d) return -1;
    return static_cast<int64_t>(vc_offset(j, c, m, d));
}

kvc_status kvc_unpack_values(const void *Vc, void *dense, int64_t records, int32_t m, int32_t d, int32_t dtype,
                             void *stream)
{
    if (!Vc || !dense) return KVC_ERR_NULL;
    if (dtype != KVC_F32 && dtype != KVC_BF16) return KVC_ERR_DTYPE;
    if (records < 0 || records > 0x7fffffff || m < 1 || d < 1) return KVC_ERR_SHAPE;
    if (!aligned16(Vc) || !aligned16(dense)) return KVC_ERR_ALIGN;
    if (records == 0) return KVC_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == KVC_F32)
        unpack_values<float><<<static_cast<unsigned>(records), 256, 0, st>>>(static_cast<const float *>(Vc), static_cast<float *>(dense), m, d);
    else
        unpack_values<uint16_t><<<static_cast<unsigned>(records), 256, 0, st>>>(static_cast<const uint16_t *>(Vc), static_cast<uint16_t *>(dense), m, d);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_HIP;
}

// ---- decode without a workspace argument, for callers that cannot allocate ------------------------
namespace {
constexpr size_t kStaticScratchBytes = static_cast<size_t>(32) << 20;
// Scratch memory of kvc_reconstruct_attend_decode_static.  Every GPU the library runs on holds its
// own copy of this array, at its own address, until the process ends.  In host code the name below
// is only a handle for hipGetSymbolAddress: kernels and copies get the address that call returns.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// address of `scratch` on the current device; asked of the runtime once per device
void *static_scratch_ptr()
{
    static std::mutex mu;
    static void *ptr[kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        ptr[dev] = p;
    }
    return ptr[dev];
}
}  // namespace

size_t kvc_static_scratch_bytes(void) { return kStaticScratchBytes; }

kvc_status kvc_reconstruct_attend_decode_static(const kvc_shape *shape, const kvc_params *params,
                                                const void *q, const void *Kc, const void *Vc,
                                                void *K_text, void *V_text, int32_t text_len,
                                                int32_t text_cap, const void *k_new, const void *v_new,
                                                float softmax_scale, void *out, float *lse_out,
                                                void *stream)
{
    // every argument check first, with a stand-in for the workspace address
    DecodeCall c;
    kvc_status st = prepare_decode(c, shape, params, q, Kc, Vc, K_text, V_text, text_len, text_cap,
                                   k_new, v_new, softmax_scale, out, lse_out,
                                   reinterpret_cast<void *>(static_cast<uintptr_t>(256)), kStaticScratchBytes, stream);
    if (st != KVC_OK) return st;
    if (kvc_workspace_bytes(shape, text_cap) > kStaticScratchBytes) return KVC_ERR_WORKSPACE;
    c.ws = static_scratch_ptr();
    if (!c.ws) return KVC_ERR_HIP;
    return dispatch_decode(c);
}

namespace {
// the shape-agnostic decode kernels serve the full cache as a call without vision tokens
kvc_shape text_only_shape(int32_t B, int32_t Hq, int32_t Hkv, int32_t d, int32_t dtype)
{
    kvc_shape s;
    s.batch = B; s.n_q_heads = Hq; s.n_kv_heads = Hkv; s.head_dim = d;
    s.n_img_tokens = 1; s.n_images = 0; s.m = 1; s.dtype = dtype;
    return s;
}
}  // namespace

size_t kvc_attend_full_workspace_bytes(int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                       int32_t head_dim, int32_t dtype, int32_t max_kv_len)
{
    const kvc_shape s = text_only_shape(batch, n_q_heads, n_kv_heads, head_dim, dtype);
    if (check_shape(&s) != KVC_OK || max_kv_len < 1) return 0;
    size_t need = generic_decode_ws_bytes(s, max_kv_len);
    if (fast_full_supported(dtype, head_dim, n_q_heads / n_kv_heads))
        need = std::max(need, fast_full_ws_bytes(batch, n_q_heads, n_kv_heads));
    return need;
}

kvc_status kvc_attend_full_decode(int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                  int32_t dtype, const void *q, void *K, void *V, int64_t stride_b,
                                  int64_t stride_h, int64_t stride_s, int32_t kv_len, int32_t kv_cap,
                                  const void *k_new, const void *v_new, float softmax_scale, void *out,
                                  float *lse_out, void *workspace, size_t workspace_bytes, void *stream)
{
    const kvc_shape s = text_only_shape(batch, n_q_heads, n_kv_heads, head_dim, dtype);
    kvc_status st = check_shape(&s);
    if (st != KVC_OK) return st;
    if (!q || !out || !K || !V) return KVC_ERR_NULL;
    if (kv_cap < 1 || kv_len < 0 || kv_len > kv_cap) return KVC_ERR_SHAPE;
    if ((k_new == nullptr) != (v_new == nullptr)) return KVC_ERR_NULL;
    if (k_new && kv_len + 1 > kv_cap) return KVC_ERR_SHAPE;
    const int32_t t = kv_len + (k_new ? 1 : 0);
    if (t == 0) return KVC_ERR_SHAPE;                               // softmax over no key
    if (!(softmax_scale >= 0.f) || isinf(softmax_scale)) return KVC_ERR_SHAPE;
    if (stride_s < head_dim || stride_h < 0 || stride_b < 0) return KVC_ERR_SHAPE;
    if (stride_s % 8 || stride_h % 8 || stride_b % 8) return KVC_ERR_ALIGN;
    if (!aligned16(q) || !aligned16(out) || !aligned16(K) || !aligned16(V) || !aligned16(k_new) ||
        !aligned16(v_new) || (reinterpret_cast<uintptr_t>(lse_out) & 3u))
        return KVC_ERR_ALIGN;
    if (!workspace) return KVC_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return KVC_ERR_ALIGN;
    const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf(static_cast<float>(head_dim));
    if (fast_full_supported(dtype, head_dim, n_q_heads / n_kv_heads)) {
        FullCall c;
        c.B = batch; c.Hq = n_q_heads; c.Hkv = n_kv_heads;
        c.q = q; c.K = K; c.V = V;
        c.sb = stride_b; c.sh = stride_h; c.ss = stride_s;
        c.t = t; c.t_in = kv_len;
        c.k_new = k_new; c.v_new = v_new;
        c.scale = scale; c.out = out; c.lse = lse_out;
        c.ws = workspace; c.ws_bytes = workspace_bytes;
        c.stream = static_cast<hipStream_t>(stream);
        c.cus = 0;
        return fast_full_decode(c);
    }
    // scalar kernels: dense cache only
    if (stride_s != head_dim || stride_h != static_cast<int64_t>(kv_cap) * head_dim ||
        stride_b != stride_h * n_kv_heads)
        return KVC_ERR_UNSUPPORTED;
    DecodeCall c;
    c.s = s;
    c.theta = q; c.U = q; c.mu = q;          // never multiplied by anything but zero without vision tokens
    c.q = q; c.Kc = q; c.Vc = q;
    c.Kt = K; c.Vt = V;
    c.t = t; c.t_in = kv_len; c.cap = kv_cap;
    c.k_new = k_new; c.v_new = v_new;
    c.scale = scale; c.out = out; c.lse = lse_out;
    c.ws = workspace; c.ws_bytes = workspace_bytes;
    c.stream = static_cast<hipStream_t>(stream);
    return generic_decode(c);
}

void kvc_dev_full_decode_chunk_steps(int32_t steps) { full_decode_set_chunk_steps(steps); }

void kvc_dev_decode_knobs(int32_t row_tiles, int32_t separate, int32_t wait_ticks)
{
    fast_decode_knobs(row_tiles, separate, wait_ticks);
}

int64_t kvc_dev_decode_fallbacks(void) { return fast_decode_fallbacks(); }

void kvc_dev_stream_decode(int32_t mode) { stream_decode_knob(mode); }

int64_t kvc_dev_stream_calls(void) { return stream_decode_calls(); }

void kvc_dev_compress_knobs(int32_t waves, int32_t jt) { fast_compress_knobs(waves, jt); }



namespace {
__global__ __launch_bounds__(256) void probe_read(const uint4 *__restrict__ p, size_t n16, unsigned *sink)
{
    size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    unsigned acc = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
        acc += a.x ^ b.y ^ c.z ^ d.w;
    }
    for (; i < n16; i += stride) acc += p[i].x;
    if (acc == 0x12345678u) *sink = acc;
}
}  // namespace

kvc_status kvc_probe_read(const void *buf, size_t bytes, void *sink, void *stream)
{
    if (!buf || !sink) return KVC_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(buf) & 15) || (bytes & 15) || (reinterpret_cast<uintptr_t>(sink) & 3))
        return KVC_ERR_ALIGN;
    if (bytes == 0) return KVC_OK;
    probe_read<<<256 * 16, 256, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const uint4 *>(buf), bytes / 16, static_cast<unsigned *>(sink));
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_HIP;
}

const char *kvc_status_string(int32_t status)
{
    switch (status) {
    case KVC_OK: return "ok";
    case KVC_ERR_NULL: return "a required pointer is NULL";
    case KVC_ERR_SHAPE: return "size or index out of range or inconsistent";
    case KVC_ERR_DTYPE: return "unknown element type";
    case KVC_ERR_ALIGN: return "pointer or stride not aligned as required";
    case KVC_ERR_WORKSPACE: return "workspace missing or too small";
    case KVC_ERR_UNSUPPORTED: return "valid but unsupported shape";
    case KVC_ERR_HIP: return "HIP runtime error at launch";
    default: return "unknown status";
    }
}

const char *kvc_version(void) { return "0.4"; }        // 0.3, 0.4: kvc_params grew by theta_packed, U_packed

}  // extern "C"
