// Full-cache ("All KV") decode attention for gfx950: bf16 storage, head_dim 128.
//
// This is the comparison point of the paper's efficiency analysis (Sec. 4; the "All KV" rows of
// Fig. 5): the same decode step as kvc_reconstruct_attend_decode, but over the UNCOMPRESSED cache --
// one new query token per sequence attends every cached key (vision and text alike) and the new
// token's own k, v, which are appended first.  It is a plain split-KV flash decode:
//
//   full_split     one workgroup per (batch element, KV head, split of the cache rows).  Each of its
//                  four waves walks its own 32-row groups of the split with its own online softmax
//                  (running maximum, running sum, un-normalised output in MFMA accumulators):
//                  logits S = sigma K q^T by 16x16x32 MFMA with the key rows as A operand straight
//                  from memory; P = exp(S - max) stays in registers and is the B operand of the
//                  second product as it comes out of the first (the 32 rows of a step are numbered
//                  the same way on both sides of the contraction); the value rows are transposed
//                  through a wave-private LDS tile to become its A operand.  The next step's rows
//                  are requested before the current step is multiplied.  The four waves merge
//                  through LDS into one part record.
//   finalize       the parts of a (batch element, query head) are merged by the finalize kernel of
//                  the capsule path (a lane per part, shuffles only).
//
// Bound: HBM (2 B H_kv (S + 1) d 2 bytes are read once; 4 flop per byte).
#include "kvc_internal.h"

#include <algorithm>

namespace kvc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int D = 128;            // head_dim of this path
constexpr int kRW = 32;           // cache rows per wave and step (one k-step of the second product)
constexpr int kWaves = 4;
constexpr int kStep = kRW * kWaves;   // rows per workgroup and step
constexpr int kLDW = 18;          // 32-bit words per channel of the transposed value tile: 16 row pairs + 2
constexpr int kLDF = D + 4;       // floats per head row of a wave's output in LDS
constexpr int kMaxSplits = 64;    // the finalize kernel keeps one part per lane

struct FullPlan {
    int Hq, Hkv, G, NS, chunk, nit, t, t_in, rec;
    unsigned qNS, qHkv;
    long sb, sh, ss;              // element strides of the cache
    float scale;
    float *Ypart;
};

__device__ inline int quot(int x, unsigned q) { return q ? static_cast<int>(__umulhi(static_cast<unsigned>(x), q)) : x; }
inline unsigned quot_multiplier(int d) { return d > 1 ? static_cast<unsigned>((1ull << 32) / static_cast<unsigned>(d)) + 1u : 0u; }
__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__global__ __launch_bounds__(64 * kWaves) void full_split(const uint16_t *__restrict__ q, uint16_t *__restrict__ K,
                                                           uint16_t *__restrict__ V, const uint16_t *__restrict__ k_new,
                                                           const uint16_t *__restrict__ v_new, FullPlan p)
{
    static_assert(D * kLDW >= 16 * kLDF, "a wave's output rows reuse its value tile");
    __shared__ __align__(16) uint32_t sVt[kWaves][D * kLDW];
    __shared__ float sM[kWaves][16], sL[kWaves][16];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, kg = lane >> 4;
    const int bh = quot(blockIdx.x, p.qNS), s = blockIdx.x - bh * p.NS;
    const int b = quot(bh, p.qHkv), h = bh - b * p.Hkv;
    const int lo = s * p.chunk, hi = min(p.t, lo + p.chunk);       // hi > lo: NS = ceil(t / chunk)
    uint16_t *Kb = K + b * p.sb + h * p.sh;
    uint16_t *Vb = V + b * p.sb + h * p.sh;
    const bool fresh = k_new != nullptr;                            // row t_in comes from k_new / v_new
    const uint16_t *kn = k_new + static_cast<size_t>(bh) * D, *vn = v_new + static_cast<size_t>(bh) * D;

    // rows of one step: key rows as MFMA A operands (lane = row r16 of a 16-row tile, 16 bytes of
    // each 64-byte k-step), value rows coalesced (16 lanes per row, a lane takes a pair of rows).
    // No test around a load: rows beyond the split are clamped to its last row.
    auto load_tile = [&](int it, u32x4 (&kf)[2][4], u32x4 (&vf)[4][2]) {
        const int r0 = lo + kStep * it + kRW * wave;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            const int x = min(r0 + 16 * tt + r16, hi - 1);
            const uint16_t *krow = (fresh && x == p.t_in) ? kn : Kb + x * p.ss;
            const u32x4 *kp = reinterpret_cast<const u32x4 *>(krow) + kg;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) kf[tt][ks] = kp[4 * ks];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int x = min(r0 + 2 * (kg + 4 * k) + e, hi - 1);
                const uint16_t *vrow = (fresh && x == p.t_in) ? vn : Vb + x * p.ss;
                vf[k][e] = *(reinterpret_cast<const u32x4 *>(vrow) + r16);
            }
    };

    u32x4 kA[2][4], vA[4][2], kB[2][4], vB[4][2];
    load_tile(0, kA, vA);
    u32x4 qf[4];
    {
        const u32x4 *qp = reinterpret_cast<const u32x4 *>(q + (static_cast<size_t>(b) * p.Hq + h * p.G + min(r16, p.G - 1)) * D) + kg;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qf[ks] = qp[4 * ks];
    }

    // online softmax state of head r16 (columns beyond the group repeat head G-1), the same in the
    // four lanes kg of a head except for the partial sum
    float m_run = -INFINITY, l_run = 0.f;
    f32x4 acc[D / 16];
#pragma unroll
    for (int ct = 0; ct < D / 16; ++ct) acc[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
    uint32_t *vt = sVt[wave];

    auto compute = [&](int it, const u32x4 (&kf)[2][4], const u32x4 (&vf)[4][2]) {
        const int r0 = lo + kStep * it + kRW * wave;
        // value rows -> LDS, transposed: rows (2 pair, 2 pair + 1) of a channel share one word
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int pair = kg + 4 * k;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t a = vf[k][0][j], c2 = vf[k][1][j];
                vt[(8 * r16 + 2 * j) * kLDW + pair] = (a & 0xffffu) | (c2 << 16);
                vt[(8 * r16 + 2 * j + 1) * kLDW + pair] = (a >> 16) | (c2 & 0xffff0000u);
            }
        }
        // logits of rows r0 + 16 tt + 4 kg + e for head r16
        float sc[2][4];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kf[tt][ks]), as_bf16x8(qf[ks]), a, 0, 0, 0);
#pragma unroll
            for (int e = 0; e < 4; ++e) sc[tt][e] = (r0 + 16 * tt + 4 * kg + e < hi) ? a[e] * p.scale : -INFINITY;
        }
        float mx = fmaxf(fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3])),
                         fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float mref = m_new == -INFINITY ? 0.f : m_new;     // nothing valid so far: exp(-inf - 0) = 0
        const float alpha = __expf(m_run - mref);
        m_run = m_new;
        uint32_t pb[2][4];
        float ls = 0.f;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                pb[tt][e] = f32_to_bf16_bits(__expf(sc[tt][e] - mref));
                ls += __uint_as_float(pb[tt][e] << 16);
            }
        l_run = l_run * alpha + ls;
        // P as B operand: position 8 kg + 4 tt + e of the k-step stands for row 16 tt + 4 kg + e
        const bf16x8 pfrag = as_bf16x8(u32x4{pb[0][0] | (pb[0][1] << 16), pb[0][2] | (pb[0][3] << 16),
                                             pb[1][0] | (pb[1][1] << 16), pb[1][2] | (pb[1][3] << 16)});
        // the wave reads back what its own lanes stored: LDS works through a wave's requests in order
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int ct = 0; ct < D / 16; ++ct) {
            const uint32_t *vr = vt + (16 * ct + r16) * kLDW + 2 * kg;
            const u32x2 v0 = *reinterpret_cast<const u32x2 *>(vr), v1 = *reinterpret_cast<const u32x2 *>(vr + 8);
            f32x4 o = acc[ct];
            o[0] *= alpha; o[1] *= alpha; o[2] *= alpha; o[3] *= alpha;
            acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(u32x4{v0[0], v0[1], v1[0], v1[1]}), pfrag, o, 0, 0, 0);
        }
        __builtin_amdgcn_wave_barrier();
    };

    // two steps per round, so that the two register sets swap by name; a step beyond the split is
    // all masked (its loads repeat the split's last row)
    for (int it = 0; it < p.nit; it += 2) {
        load_tile(it + 1, kB, vB);
        compute(it, kA, vA);
        load_tile(it + 2, kA, vA);
        compute(it + 1, kB, vB);
    }

    // ---- the four waves merge into one part record ------------------------------------------------
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    float *fo = reinterpret_cast<float *>(vt);                     // [16 heads][kLDF]
#pragma unroll
    for (int ct = 0; ct < D / 16; ++ct) *reinterpret_cast<f32x4 *>(fo + r16 * kLDF + 16 * ct + 4 * kg) = acc[ct];
    if (kg == 0) { sM[wave][r16] = m_run; sL[wave][r16] = l_run; }
    __syncthreads();
    float *yp = p.Ypart + (static_cast<size_t>(bh) * p.NS + s) * p.rec;
    for (int idx = threadIdx.x; idx < p.G * (D / 4); idx += 64 * kWaves) {
        const int g = idx / (D / 4), c4 = (idx - g * (D / 4)) * 4;
        const float M = fmaxf(fmaxf(sM[0][g], sM[1][g]), fmaxf(sM[2][g], sM[3][g]));
        const float mref = M == -INFINITY ? 0.f : M;
        f32x4 y = {0.f, 0.f, 0.f, 0.f};
        float l = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float a = __expf(sM[w][g] - mref);
            const f32x4 o = *reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(sVt[w]) + g * kLDF + c4);
            y[0] += a * o[0]; y[1] += a * o[1]; y[2] += a * o[2]; y[3] += a * o[3];
            l += a * sL[w][g];
        }
        *reinterpret_cast<f32x4 *>(yp + g * D + c4) = y;
        if (c4 == 0) {
            yp[p.G * D + g] = M;
            yp[p.G * D + p.G + g] = l;
        }
    }
    // the cache grows as in the backbone: the split that owns row t_in stores the new token
    if (fresh && p.t_in >= lo && p.t_in < hi && threadIdx.x < 32) {
        const int half = threadIdx.x >> 4, piece = threadIdx.x & 15;
        const uint16_t *src = half ? vn : kn;
        uint16_t *dst = (half ? Vb : Kb) + p.t_in * p.ss;
        *(reinterpret_cast<u32x4 *>(dst) + piece) = *(reinterpret_cast<const u32x4 *>(src) + piece);
    }
}

int g_chunk_steps = 0;            // developer knob: steps of 128 rows per split (0: chosen by the rule below)

FullPlan make_full_plan(const FullCall &c, void *ws)
{
    FullPlan p;
    p.Hq = c.Hq; p.Hkv = c.Hkv; p.G = c.Hq / c.Hkv;
    p.t = c.t; p.t_in = c.t_in;
    p.sb = c.sb; p.sh = c.sh; p.ss = c.ss;
    p.scale = c.scale;
    // Rows per split: enough splits to give every CU about two workgroups (the rows of a split are
    // read by one workgroup, 64 KB in flight per step), never more than the finalize kernel's 64 parts
    const int steps_total = (c.t + kStep - 1) / kStep;
    const long bh = static_cast<long>(c.B) * c.Hkv;
    int cs = g_chunk_steps;
    if (cs <= 0) {
        const long want = std::max(1L, (2L * c.cus + bh - 1) / bh);        // splits per (b, head)
        cs = static_cast<int>((steps_total + want - 1) / want);
        if (cs < 2) cs = steps_total >= 2 ? 2 : 1;
    }
    while ((steps_total + cs - 1) / cs > kMaxSplits) ++cs;
    p.chunk = cs * kStep;
    p.nit = std::min(cs, steps_total);
    p.NS = (c.t + p.chunk - 1) / p.chunk;
    p.rec = static_cast<int>(align_up(static_cast<size_t>(p.G) * D + 2 * p.G, 4));
    p.qNS = quot_multiplier(p.NS);
    p.qHkv = quot_multiplier(p.Hkv);
    p.Ypart = static_cast<float *>(ws);
    return p;
}

}  // namespace

void full_decode_set_chunk_steps(int steps) { g_chunk_steps = steps; }

bool fast_full_supported(int dtype, int head_dim, int G) { return dtype == KVC_BF16 && head_dim == D && G >= 1 && G <= 16; }

size_t fast_full_ws_bytes(int B, int Hq, int Hkv)
{
    const int G = Hq / Hkv;
    return static_cast<size_t>(B) * Hkv * kMaxSplits * align_up(static_cast<size_t>(G) * D + 2 * G, 4) * sizeof(float);
}

kvc_status fast_full_decode(const FullCall &c)
{
    if (fast_full_ws_bytes(c.B, c.Hq, c.Hkv) > c.ws_bytes) return KVC_ERR_WORKSPACE;
    FullCall cc = c;
    if (cc.cus <= 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        cc.cus = cus;
    }
    const FullPlan p = make_full_plan(cc, c.ws);
    // quot(): workgroup ids divided by NS, (b, head) ids by H_kv
    if (static_cast<long>(c.B) * c.Hkv * p.NS * std::max(p.NS, c.Hkv) >= (1ll << 32)) return KVC_ERR_UNSUPPORTED;
    full_split<<<c.B * c.Hkv * p.NS, 64 * kWaves, 0, c.stream>>>(
        static_cast<const uint16_t *>(c.q), static_cast<uint16_t *>(c.K), static_cast<uint16_t *>(c.V),
        static_cast<const uint16_t *>(c.k_new), static_cast<const uint16_t *>(c.v_new), p);
    if (hipGetLastError() != hipSuccess) return KVC_ERR_HIP;
    // no vision parts: the finalize kernel's "+ (sum P_vis) mu" term is zero; q stands in for mu
    // (at least H_kv d finite values)
    return finalize_parts(p.Ypart, p.NS, 0, p.rec, c.B, c.Hq, c.Hkv, c.q, c.out, c.lse, c.stream);
}

}  // namespace kvc
