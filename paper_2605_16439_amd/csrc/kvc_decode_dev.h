// Device-side declarations shared by the decode kernels of libkvcapsule.so (kvc_fast_decode.hip,
// kvc_stream_decode.hip, kvc_full_decode.hip): register image types, index helpers, the decode plan, and text_part --
// the complete attention part of 128 rows of the text cache, which the four-kernel decode and the
// full-cache decode run as extra workgroups.  Nothing here is part of the C ABI.
#pragma once
#include "kvc_internal.h"

namespace kvc {
namespace dd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
// 16-byte and 8-byte register images as native vectors (HIP's uint4 / float2 structs turn plain
// copies into memcpy through private memory, which ends up in scratch)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));     // a 16-byte access at a dword-aligned address
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int D = 128;          // head_dim of this path
constexpr int kRB = 128;        // query rows are padded to this: fb_probs workgroups take 64 or 128 (4 or 8 waves)
constexpr int kPC = 64;         // positions per fb_probs workgroup (one softmax tile)
constexpr int kTPW = 2;         // 16-row key tiles per wavefront in fa_scores
constexpr int kJC = 64;         // capsule rows per fc_fused workgroup (one 16-row tile per wave)
constexpr int kXC = 128;        // text rows per fa_scores text workgroup
constexpr int kMaxParts = 256;  // fd_finalize keeps one scale per part in LDS
constexpr int kSWLD = kXC + 8;  // padded row (bf16) of the text probabilities in LDS
constexpr int kLDV = kXC + 8;   // padded row (bf16) of the transposed text values in LDS
constexpr int kWLD = kJC + 8;   // padded row (bf16) of the W tile in LDS
constexpr size_t kLdsBudget = 150 * 1024;
constexpr int kCtrStride = 16;  // 64-bit words per arrival counter: one counter per 128-byte line
constexpr int kMaxFlags = 512;  // arrival counters at the start of the workspace
constexpr int kDenseRows = 24;  // "image blocks per 64-row block" = 2^24: the dense layout of the query rows

struct Plan {
    int B, Hq, Hkv, G, n, I, m, t, t_in, cap;
    int R, R_pad, NRB, RBW, m_pad, m16, NC;   // RBW: waves (16-row tiles) per fb_probs workgroup
    int UPBs, RV;                   // log2 of the image blocks per 64-row block of query rows; valid rows of a full block
    int fab;                        // fa_scores and fb_probs run as one launch (fab_fused)
    int wait_ticks;                 // fab_fused: how long a workgroup waits for its siblings (10 ns units)
    unsigned epoch;                 // fab_fused: this call's number; counter words of another epoch count as zero
    unsigned long long *flags;      // fab_fused: [Hkv NRB] arrival counters (epoch, count) at the start of the workspace
    unsigned *fallbacks;            // fab_fused: debug counter of workgroups that computed alone (may be null)
    int tiles_per_unit, vis_tiles, nvis_a, ntext_a;   // fa_scores: vision workgroups, text workgroups (these come first)
    int ntext_c;                    // fc_fused: text workgroups (the highest ids)
    int UP, NT, NG, JS, NXC, nparts, rec;
    int merge, nvp;                 // one part per workgroup (its image blocks merged); vision parts per (b, head)
    // ragged batch (kernels instantiated with RAG = true): n_img[b] image blocks, tlen[b] text rows before the
    // call; I, t and t_in are then the largest values a sequence may have.  Null in a uniform call.
    const int32_t *n_img, *tlen;
    int nvis_b, nvis_c;
    // multipliers for the divisions by NXC, Hkv, tiles_per_unit, I, NC, JS and G (see quot())
    unsigned qNXC, qHkv, qTPU, qI, qNC, qJS, qG;
    float scale;
#if defined(KVC_TIMELINE)
    unsigned long long *tl;         // timeline slots, see TS()
#endif
    uint16_t *S;
    uint16_t *P;
    f32x2 *stats;
    float *Ypart;
    size_t bytes;
};

// Developer aid, compiled in only with -DKVC_TIMELINE: thread 0 of every workgroup records the
// wall clock at a few points of each kernel (kernel id, slot) in the last MiB of the workspace.
#if defined(KVC_TIMELINE)
#define TS(KID, K)                                                                        \
    do {                                                                                  \
        if (p.tl && threadIdx.x == 0)                                                     \
            p.tl[((KID) * 1024 + (blockIdx.x < 1024 ? blockIdx.x : 1023)) * 8 + (K)] = wall_clock64(); \
    } while (0)
constexpr size_t kTimelineBytes = 1 << 20;
#else
#define TS(KID, K) do { } while (0)
constexpr size_t kTimelineBytes = 0;
#endif

// ---- arrival counters in the caller's workspace ------------------------------------------------------
// A counter word carries (epoch, count), the epoch in the upper half.  The epoch is a number the host draws
// per call from a counter that only grows, and a finished call leaves zeros behind.  Before a workgroup adds
// to a word it raises it to (epoch, 0) with an atomic maximum: a word left by an earlier call (zero, or an
// older epoch after a failed call) becomes (epoch, 0); a word that already carries this epoch keeps its
// count -- in whatever order the workgroups get there.  Only "all arrived" under the call's own epoch ends a
// wait.  Memory that holds something else (a fresh allocation, another kernel's data) usually reads as a
// LARGER epoch: the maximum leaves it alone, nobody ever sees this call's epoch, every workgroup gives up
// waiting after wait_ticks and computes alone (correct, slower), and the call's last kernel writes zeros,
// so the next call is at full speed.
typedef unsigned long long u64;
__device__ inline u64 ctr_word(unsigned epoch, unsigned count) { return (static_cast<u64>(epoch) << 32) | count; }
// the word as the L2 holds it: an atomic add of zero is carried out there (a plain load may be answered
// by the CU's L1); waits for the answer
__device__ inline u64 ctr_peek(u64 *w)
{
    u64 seen;
    asm volatile("global_atomic_add_x2 %0, %1, %2, off sc0\n\ts_waitcnt vmcnt(0)" : "=&v"(seen) : "v"(w), "v"(static_cast<u64>(0)) : "memory");
    return seen;
}
// nothing is waited for: the caller's next "all my stores are done" point covers it
__device__ inline void ctr_claim(u64 *w, unsigned epoch)
{
    __hip_atomic_fetch_max(w, ctr_word(epoch, 0u), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// x / d for 0 <= x with x d < 2^32, as one multiplication by q = floor(2^32 / d) + 1 (q = 0 stands
// for d = 1).  The index arithmetic at the top of every kernel sits in front of its first load; a
// division by a run-time value costs some thirty dependent instructions there.
__device__ inline int quot(int x, unsigned q) { return q ? static_cast<int>(__umulhi(static_cast<unsigned>(x), q)) : x; }
inline unsigned quot_multiplier(int d) { return d > 1 ? static_cast<unsigned>((1ull << 32) / static_cast<unsigned>(d)) + 1u : 0u; }

// Where the arguments are not preloaded (fd_finalize): the plan and the pointers after it span two
// 128-byte lines of device memory that no cache holds when a workgroup starts.  Naming one value of
// each line at the top of the kernel makes the compiler fetch both at once, before the first test
// that could end the workgroup, instead of paying one memory round trip after the other; naming what
// the address arithmetic in front of the first loads needs keeps those fetches in the same batch.
#define KVC_FETCH_ARGS(first, last, a, b, c, d, e, f) \
    asm volatile("" ::"s"(first), "s"(last), "s"(a), "s"(b), "s"(c), "s"(d), "s"(e), "s"(f))

// Makes the compiler fetch the named arguments (those that are not preloaded) here, in one batch:
// placed behind the first vector loads, their round trip to device memory hides behind those loads
// instead of standing in front of the first use of each.
template <class T> __device__ __forceinline__ void fetch_one(T v) { asm volatile("" ::"s"(v)); }
template <class... T> __device__ __forceinline__ void fetch_now(T... v) { (fetch_one(v), ...); }

__host__ __device__ inline u32x4 u32x4_mk(unsigned a, unsigned b, unsigned c, unsigned d) { return u32x4{a, b, c, d}; }
__host__ __device__ inline u32x2 u32x2_mk(unsigned a, unsigned b) { return u32x2{a, b}; }
__host__ __device__ inline f32x4 f32x4_mk(float a, float b, float c, float d) { return f32x4{a, b, c, d}; }
__host__ __device__ inline f32x2 f32x2_mk(float a, float b) { return f32x2{a, b}; }
__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ inline float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
// element (channel c, row x) of the transposed text-value tile; the 16-byte chunks of a channel
// row are XOR-swizzled with the index of the channel's 16-row MFMA tile: the transposing stores
// spread over the banks and the operand reads of one tile stay conflict-free
__device__ inline int vt_index(int c, int x) { return c * kLDV + ((((x >> 3) ^ (c >> 4)) & (kXC / 8 - 1)) << 3) + (x & 7); }

// first query row of image block ub (b*I + i) of a KV head
__host__ __device__ inline int unit_row(int ub, int UPBs, int G) { return ((ub >> UPBs) << 6) + (ub & ((1 << UPBs) - 1)) * G; }
// rows of a 64-row block beyond its image blocks, and rows beyond the last image block, hold nothing
__device__ inline bool row_valid(const Plan &p, int r) { return (r & 63) < p.RV && r < p.R; }

// ------------------------------------------------------------------------------------------
// text_part: the complete attention part of kXC rows of the text cache of one (batch, KV head),
// by four waves; `id` numbers the chunks, `lds` holds kTextLds bytes.  Runs as extra workgroups of
// fc_fused (its longest launch, bound by the L2s, with CUs and HBM bandwidth to spare), or of
// fa_scores when there are no vision tokens.
// Part record in Ypart: [G][D] floats of un-normalised output, [G] maxima, [G] sums.
// ------------------------------------------------------------------------------------------
constexpr size_t kTextLds = (16 * kSWLD + D * kLDV) * sizeof(uint16_t) + 2 * 4 * 16 * sizeof(float);

// GT: the group size, or 0 to take it from the plan.  RAG: per-sequence text lengths (ragged batch).  tid: the thread's index within the four waves
// that work on this chunk (a workgroup of eight waves runs two chunks side by side, each half with
// its own `lds`; both halves meet the same barriers).  live = false: the chunk is a stand-in that
// keeps a half in step with the other one's barriers; nothing is stored.
template <int GT, bool RAG>
__device__ __forceinline__ void text_part(const Plan &p, const uint16_t *__restrict__ q, uint16_t *__restrict__ Kt,
                                          uint16_t *__restrict__ Vt, const uint16_t *__restrict__ k_new,
                                          const uint16_t *__restrict__ v_new, uint16_t *lds, const int id,
                                          const int tid, const bool live)
{
    const int G = GT ? GT : p.G;
    fetch_now(p.qNXC, p.NXC, p.qHkv, p.Hkv, p.Hq, p.t, p.t_in, p.cap, q, Kt, Vt, k_new, v_new, p.scale, p.Ypart, p.nparts,
              p.nvp, p.rec, p.tlen);
    const int wave = tid >> 6, lane = tid & 63;
    const int r16 = lane & 15, kg = lane >> 4;
    // ---------------- text rows: one chunk of kXC rows of one (batch, KV head) ----------------
    uint16_t (*sWb)[kSWLD] = reinterpret_cast<uint16_t (*)[kSWLD]>(lds);               // probabilities [head][row], bf16
    uint16_t *sVt = lds + 16 * kSWLD;                                                  // V^T [channel][row]
    float (*sRed)[4][16] = reinterpret_cast<float (*)[4][16]>(lds + 16 * kSWLD + D * kLDV);   // per-wave maxima / sums per head
    const int bh = quot(id, p.qNXC), xc = id - bh * p.NXC;
    const int b = quot(bh, p.qHkv), h = bh - b * p.Hkv;
    const bool fresh = k_new != nullptr;                       // row t_in comes from k_new / v_new
    // this sequence's rows: t_in before the call (the new token goes there), t attended
    // (RAG: a ragged batch, the sequence's own count is read; otherwise the call's values, at no cost)
    int t_in = p.t_in, t = p.t;
    if constexpr (RAG) {
        const int tlb = max(p.tlen[b], 0);
        t_in = min(tlb, p.t_in);
        t = fresh ? t_in + 1 : min(tlb, p.t);
    }
    // a chunk beyond the sequence's rows keeps lo = hi: every load is clamped to a valid row, every logit masked
    const int lo = xc * kXC, hi = max(min(t, lo + kXC), lo);
    const int xlast = max(min(hi, t) - 1, 0);                 // the last row the chunk (or, if it is empty, the sequence) has
    // value rows of the chunk (16 lanes per row, a lane takes pairs of consecutive rows) and key
    // rows of this wave's two 16-row tiles
    const int rowl = wave * 4 + kg, cs = r16;
    u32x4 vb[kXC / 32][2], kf[2][4], qf[4];
#pragma unroll
    for (int it = 0; it < kXC / 32; ++it)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int x = min(lo + 2 * (rowl + 16 * it) + e, xlast);
            const uint16_t *vrow = (fresh && x == t_in) ? v_new + static_cast<size_t>(bh) * D
                                                          : Vt + (static_cast<size_t>(bh) * p.cap + x) * D;
            vb[it][e] = *(reinterpret_cast<const u32x4 *>(vrow) + cs);
        }
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        const int x = min(lo + 32 * wave + 16 * tt + r16, xlast);
        const uint16_t *krow = (fresh && x == t_in) ? k_new + static_cast<size_t>(bh) * D
                                                      : Kt + (static_cast<size_t>(bh) * p.cap + x) * D;
        const u32x4 *kp = reinterpret_cast<const u32x4 *>(krow) + kg;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) kf[tt][ks] = kp[4 * ks];
    }
    {
        const u32x4 *qp = reinterpret_cast<const u32x4 *>(q + (static_cast<size_t>(b) * p.Hq + h * G + min(r16, G - 1)) * D) + kg;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qf[ks] = qp[4 * ks];
    }
    TS(0, 1);
    // logits: lane (head r16, rows 32 wave + 16 tt + 4 kg + e) keeps 8 of them
    f32x4 sc[2];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kf[tt][ks]), as_bf16x8(qf[ks]), acc, 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            sc[tt][e] = (lo + 32 * wave + 16 * tt + 4 * kg + e < hi) ? acc[e] * p.scale : -INFINITY;
    }
    float mx = fmaxf(fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3])),
                     fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    if (kg == 0) sRed[0][wave][r16] = mx;
    // value rows -> LDS transposed: rows (x, x+1) of channel c share one 32-bit word
#pragma unroll
    for (int it = 0; it < kXC / 32; ++it) {
        const int xl2 = 2 * (rowl + 16 * it);
        const uint32_t a[4] = {vb[it][0].x, vb[it][0].y, vb[it][0].z, vb[it][0].w};
        const uint32_t c2[4] = {vb[it][1].x, vb[it][1].y, vb[it][1].z, vb[it][1].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            *reinterpret_cast<uint32_t *>(sVt + vt_index(8 * cs + 2 * e, xl2)) = (a[e] & 0xffffu) | (c2[e] << 16);
            *reinterpret_cast<uint32_t *>(sVt + vt_index(8 * cs + 2 * e + 1, xl2)) = (a[e] >> 16) | (c2[e] & 0xffff0000u);
        }
    }
    __syncthreads();
    TS(0, 2);
    // probabilities relative to the chunk's own maximum, straight from the accumulator layout
    mx = fmaxf(fmaxf(sRed[0][0][r16], sRed[0][1][r16]), fmaxf(sRed[0][2][r16], sRed[0][3][r16]));
    const float mref = mx == -INFINITY ? 0.f : mx;             // an empty chunk: all weights zero, no inf - inf
    float sm = 0.f;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        uint32_t eb[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            eb[e] = f32_to_bf16_bits(__expf(sc[tt][e] - mref));     // exp(-inf) = 0 beyond the chunk
            sm += __uint_as_float(eb[e] << 16);
        }
        *reinterpret_cast<u32x2 *>(&sWb[r16][32 * wave + 16 * tt + 4 * kg]) = u32x2_mk(eb[0] | (eb[1] << 16), eb[2] | (eb[3] << 16));
    }
    sm += __shfl_xor(sm, 16, 64);
    sm += __shfl_xor(sm, 32, 64);
    if (kg == 0) sRed[1][wave][r16] = sm;
    __syncthreads();
    TS(0, 3);
    // out_part^T[c][g] = sum_x V^T[c][x] P[g][x]; each wave owns two 16-channel tiles
    float *yp = p.Ypart + (static_cast<size_t>(bh) * p.nparts + p.nvp + xc) * p.rec;
#pragma unroll
    for (int ct2 = 0; ct2 < 2; ++ct2) {
        const int ct = 2 * wave + ct2;
        f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < kXC / 32; ++ks) {
            const bf16x8 afrag = *reinterpret_cast<const bf16x8 *>(sVt + vt_index(16 * ct + r16, 32 * ks + 8 * kg));
            const bf16x8 bfrag = *reinterpret_cast<const bf16x8 *>(&sWb[r16][32 * ks + 8 * kg]);
            o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, bfrag, o, 0, 0, 0);
        }
        if (r16 < G && live) *reinterpret_cast<f32x4 *>(yp + r16 * D + 16 * ct + 4 * kg) = o;
    }
    if (tid < G && live) {
        yp[G * D + tid] = mx;                    // lanes 0..15 of wave 0 hold the maximum of head r16
        yp[G * D + G + tid] = sRed[1][0][tid] + sRed[1][1][tid] + sRed[1][2][tid] + sRed[1][3][tid];
    }
    // Sec. 3.2: the text cache keeps growing as in the backbone -- store the new token's k, v
    if (fresh && live && t_in >= lo && t_in < hi && tid < 32) {
        const int half = tid >> 4, piece = tid & 15;
        const uint16_t *src = (half ? v_new : k_new) + static_cast<size_t>(bh) * D;
        uint16_t *dst = (half ? Vt : Kt) + (static_cast<size_t>(bh) * p.cap + t_in) * D;
        *(reinterpret_cast<u32x4 *>(dst) + piece) = *(reinterpret_cast<const u32x4 *>(src) + piece);
    }
    TS(0, 4);
}

}  // namespace dd
}  // namespace kvc
