// Decode step in one pass per workgroup ("stream" form of Alg. 1, "Fused KVCapsule"): a workgroup owns
// UP image blocks of one (batch element, KV head) and a slice of PS of the n positions, and takes its
// rows through all four products, meeting the other slices' workgroups once (the scores, which all of them
// need, are computed a share each and handed over through the L2):
//     S = sigma q Kc^T            (Alg. 1 step 1; Kc streamed once, scores kept in LDS)
//     L = S theta[:, slice]       (step 2; theta in its packed form, straight from memory into MFMA operands)
//     P = exp(L - slice max)      (softmax numerators relative to the slice's own maximum)
//     W = P U[:, slice]^T         (step 3, the part of the sum over positions that this slice holds)
//     Y = W Vc                    (step 4; by linearity the slices' partial W may be multiplied separately)
// and writes one part record (un-normalised output, maximum, sums) that the finalize kernel merges into
// the joint softmax over all slices, image blocks and text rows (Sec. 3.2: reconstructed vision KV and
// text KV go through one attention).  A share of the text rows rides along in every workgroup.
// Against the four-kernel form (kvc_fast_decode.hip) nothing crosses a kernel boundary but the part
// records; the price is that theta and U are read once per group of UP image blocks instead of once per
// 64 query rows.  Every loop of the main path has a compile-time trip count and no load sits under a
// run-time test, so the compiler's count of loads in flight stays exact and each phase's first loads are
// requested while the previous phase still computes.
#include <algorithm>
#include <atomic>

#include "kvc_decode_dev.h"

namespace kvc {

using namespace dd;

namespace {

int g_stream_mode = -1;          // developer knob: -1 built-in rule, 0 never, 1 wherever an instance exists
std::atomic<long> g_stream_calls{0};   // calls this path has taken (tests read it)

constexpr int kTT = 8;           // at most this many 16-row text tiles per workgroup (one per wavefront)
constexpr int kTX = 16 * kTT;    // text rows per workgroup
constexpr int kLTL = kTX + 4;    // padded row (floats) of the text logits in LDS

struct SPlan {
    int B, Hq, Hkv, I, n, m, t, t_in, cap;
    int IU, F, NGR, chunk;        // unit groups per sequence, slices per image block, groups, groups per XCD
    int TT;                       // 16-row text tiles per workgroup
    int nparts, rec;
    unsigned qF, qBIU, qIU;
    float scale;
    float *Ypart;
    uint16_t *Sx;                 // scores handed between the F workgroups of a group: [NGR][16][MP] bf16
    u64 *flags;                   // one arrival counter (epoch, count) per group, at the start of the workspace
    unsigned epoch;
    int wait_ticks;
    unsigned *fallbacks;
    // ragged batch (instances with RAG = true): n_img[b] image blocks, tlen[b] text rows before the call; I, t
    // and t_in are then the largest values a sequence may have.  Null in a uniform call.
    const int32_t *n_img, *tlen;
#if defined(KVC_TIMELINE)
    unsigned long long *tl;       // timeline slots, see TS()
#endif
};

// LDS barrier that leaves global loads in flight (__syncthreads() also waits for those)
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Blocked record ([rows / 8] blocks of [X][w], w = 8 or rows % 8 for the last): where lane (x, kg) finds
// its operand of the LAST k-step (blocks 4 (KS - 1) + kg), in bytes from the record's start, and by how
// much the 16-byte window must be shifted (the shorter last block is read as an aligned window around
// the lane's values).  Blocks beyond the record read a valid one: their weights are zero.
struct LastStep {
    uint32_t off;
    int ds;
    uint32_t bs;
};
__device__ __forceinline__ LastStep last_step(int rows, int X, int x, int kg, int KS)
{
    const int nfull = rows >> 3, wt = rows & 7;
    const int jbq = 4 * (KS - 1) + kg;
    const int tail_off = x * 2 * wt;
    const int a0 = max(min(tail_off & ~3, X * 2 * wt - 16), 0);
    const int sh = tail_off - a0;
    const bool mine = wt != 0 && (jbq == nfull || nfull == 0);
    const int jb = max(min(jbq, nfull - 1), 0);
    LastStep r;
    r.off = mine ? static_cast<uint32_t>(nfull * 8 * X * 2 + a0) : static_cast<uint32_t>(jb * 8 * X * 2 + x * 16);
    r.ds = mine ? sh >> 2 : 0;
    r.bs = mine ? (sh & 2) * 8u : 0u;
    return r;
}
// 128-bit right shift by ds dwords and bs bits (registers only; identity for ds = bs = 0)
__device__ __forceinline__ u32x4 shift_window(u32x4 wv, int ds, uint32_t bs)
{
    const bool d1 = ds & 1, d2 = ds & 2;
    const uint32_t y0 = d1 ? wv.y : wv.x, y1 = d1 ? wv.z : wv.y, y2 = d1 ? wv.w : wv.z, y3 = d1 ? 0u : wv.w;
    const uint32_t x0 = d2 ? y2 : y0, x1 = d2 ? y3 : y1, x2 = d2 ? 0u : y2, x3 = d2 ? 0u : y3;
    return u32x4_mk(__builtin_amdgcn_alignbit(x1, x0, bs), __builtin_amdgcn_alignbit(x2, x1, bs),
                    __builtin_amdgcn_alignbit(x3, x2, bs), x3 >> bs);
}

constexpr size_t stream_lds_bytes(int KS, int PS)
{
    return static_cast<size_t>(2 * 16 * (32 * KS + 16) + 16 * (PS + 16)) * 2 +
           static_cast<size_t>(16 * kLTL + 8 * 8 * D + 2 * 8 * 16 + 2 * 16) * 4 +
           static_cast<size_t>(8) * 16 * D * 2;                     // a 16-row tile of keys per wavefront
}

// Part record: [G][D] floats of un-normalised output, [G] maxima, [G] sums, [G] sums over vision positions.
//
// The kernel is bound by the number of instructions a wavefront issues (every byte it needs is on its way
// long before it is used), so what can be wave-uniform is kept in scalar registers -- the wavefront's index is
// read with readfirstlane, tile bases are scalar, lanes add a fixed 32-bit offset -- and clamps and masks are
// compiled only into the rounds whose tiles can reach the end of the compressed axis.
template <int G, int UP, int PS, int KS, bool RAG>
__global__ __launch_bounds__(512) void fs_stream(const uint16_t *__restrict__ q, const uint16_t *__restrict__ Kc,
                                                 const uint16_t *__restrict__ thp, const uint16_t *__restrict__ Up,
                                                 const uint16_t *__restrict__ Vc, uint16_t *__restrict__ Kt,
                                                 uint16_t *__restrict__ Vt, const uint16_t *__restrict__ k_new,
                                                 const uint16_t *__restrict__ v_new, SPlan p)
{
    constexpr int RU = UP * G;                           // query rows of the workgroup
    static_assert(RU <= 16, "the rows must fit one MFMA tile");
    constexpr int T = 2 * KS, MP = 32 * KS;              // 16-row tiles / padded length of the compressed axis
    constexpr int TI = 2 * (KS - 1);                     // tiles below this index hold rows < m only (m > 32 (KS - 1))
    constexpr int LDS = MP + 16, LDP = PS + 16;          // LDS rows 32 mod 64 bytes apart: operand reads without bank conflicts
    constexpr int NPT = PS / 16, NPW = (NPT + 7) / 8;    // position tiles, per wavefront
    constexpr int KP = PS / 32;                          // k-steps over the slice's positions
    constexpr int NI = UP * T, NRS = (NI + 7) / 8;       // key tiles, rounds of eight
    constexpr int NRW = (T + 7) / 8;                     // rounds of eight tiles of U
    constexpr int PDL = KS < 13 ? KS : 13;               // k-steps of theta requested ahead
    constexpr int PDW = NRW < 3 ? NRW : 3;               // tiles of U requested ahead
    constexpr int PDY = KS < (UP > 2 ? 2 : 6) ? KS : (UP > 2 ? 2 : 6);   // k-steps of compressed values requested ahead
    static_assert(PS % 32 == 0 && NPW <= 3, "slice of positions");

    extern __shared__ __align__(16) uint16_t dyn[];
    uint16_t *sS = dyn;                                  // scores       [16][LDS] bf16
    uint16_t *sW = sS + 16 * LDS;                        // W            [16][LDS] bf16
    uint16_t *sP = sW + 16 * LDS;                        // numerators   [16][LDP] bf16
    float *sTL = reinterpret_cast<float *>(sP + 16 * LDP);   // text logits, then weights [16][kLTL]
    float *sYt = sTL + 16 * kLTL;                        // text part of the output, per wavefront [8][8][D]
    float *sRed = sYt + 8 * 8 * D;                       // row maxima [16][8 waves], row sums [16][8 waves]
    float *sTm = sRed + 2 * 8 * 16;                      // text maxima [16], text sums [16]

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int r16 = lane & 15, kg = lane >> 4;
    // this wavefront's staging tile: 16 rows of keys (256 bytes each)
    char *sTile = reinterpret_cast<char *>(sTm + 2 * 16) + wave * (16 * D * 2);

    // workgroup -> (KV head, batch element, unit group, slice).  Ids are dealt round-robin over the 8 XCDs;
    // an XCD takes a contiguous run of groups in (head, batch element, unit group) order, all slices of a
    // group with it: the group's capsule is fetched into one L2, a head's theta and U into as few as possible.
    const int xcd = blockIdx.x & 7, kk = blockIdx.x >> 3;
    const int gl = quot(kk, p.qF), s = kk - gl * p.F;
    const int gk = xcd * p.chunk + gl;
    if (gl >= p.chunk || gk >= p.NGR) return;
    const int h = quot(gk, p.qBIU), bu = gk - h * (p.B * p.IU);
    const int b = quot(bu, p.qIU), ug = bu - b * p.IU;
    const int i0 = ug * UP, p0 = s * PS, bh = b * p.Hkv + h, pi = ug * p.F + s;
    const int m = p.m, n = p.n;
    TS(4, 0);

    // ---- request: query rows, this workgroup's share of the text rows ----------------------------------
    u32x4 qf[4];
    {
        const u32x4 *qp = reinterpret_cast<const u32x4 *>(q + (static_cast<size_t>(b) * p.Hq + h * G + min(r16, G - 1)) * D) + kg;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qf[ks] = qp[4 * ks];
    }
    const bool fresh = k_new != nullptr;
    // this sequence's counts: image blocks it has, text rows before the call (the new token goes there) and
    // attended (RAG: a ragged batch, the sequence's own counts are read; otherwise the call's values, at no cost)
    int n_img = p.I, t_in = p.t_in, t = p.t;
    if constexpr (RAG) {
        n_img = min(max(p.n_img[b], 0), p.I);
        const int tlb = max(p.tlen[b], 0);
        t_in = min(tlb, p.t_in);
        t = fresh ? t_in + 1 : min(tlb, p.t);
    }
    const int TT = p.TT, TR = 16 * TT, x0 = pi * TR;
    const int xlast = max(t - 1, 0);
    // Rows of keys are loaded whole -- 16 lanes per 256-byte row, so that a quarter-wave
    // reads contiguous lines -- and turned into MFMA operands (16 rows x 16 bytes per quarter-wave) through
    // this wavefront's LDS tile; the 16-byte pieces of row r are stored at piece ^ r, which keeps both the
    // stores and the operand reads free of bank conflicts.  (Operand-shaped loads straight from memory
    // touch 16 lines per quarter-wave and run at a fifth of the rate.)
    const int krow = lane >> 4, kpc = lane & 15;       // key tile: row within a pass of four, 16-byte piece
    // (the new token's row is not in the cache yet: its values are loaded on the side and selected in)
    const uint16_t *kn_p = fresh ? k_new + static_cast<size_t>(bh) * D : q, *vn_p = fresh ? v_new + static_cast<size_t>(bh) * D : q;
    const int t_new = fresh ? t_in : -1;
    const char *kt_base = reinterpret_cast<const char *>(Kt + static_cast<size_t>(bh) * p.cap * D);
    const char *vt_base = reinterpret_cast<const char *>(Vt + static_cast<size_t>(bh) * p.cap * D);
    u32x4 tk[4];
    const int xk0 = x0 + 16 * min(wave, max(TT - 1, 0));
#pragma unroll
    for (int i = 0; i < 4; ++i)
        tk[i] = *reinterpret_cast<const u32x4 *>(kt_base + static_cast<size_t>(min(xk0 + 4 * i + krow, xlast)) * 256 + kpc * 16);
    const u32x4 tkn = *(reinterpret_cast<const u32x4 *>(kn_p) + kpc);
    // value rows of the text share: wave w takes rows 2 TT w ... 2 TT (w + 1) - 1 (a row is wave-uniform, so
    // its clamp is scalar work); a lane two channels
    uint32_t tv[2 * kTT];
    const int xv0 = x0 + 2 * TT * wave, xvl = min(x0 + max(TR - 1, 0), xlast);
#pragma unroll
    for (int rr = 0; rr < 2 * kTT; ++rr)
        tv[rr] = *reinterpret_cast<const uint32_t *>(vt_base + static_cast<size_t>(min(xv0 + rr, xvl)) * 256 + lane * 4);
    const uint32_t tvn = *(reinterpret_cast<const uint32_t *>(vn_p) + lane);

    // ---- step 1: S = sigma q Kc^T in tiles of 16 compressed keys.  The F workgroups of a group need the same
    // scores: each computes the tiles of its own share and hands them to the others through the L2 (they run on
    // one XCD), so that a workgroup pulls a quarter of the group's keys through its L1 at memory's latency
    // instead of all of them.
    const char *kc_base = reinterpret_cast<const char *>(Kc + (static_cast<size_t>(bh) * p.I + i0) * m * D);
    constexpr int FS = 1024 / PS;                          // shares = slices per image block (instances exist for n = 1024)
    constexpr int QI = (NI + FS - 1) / FS, NRQ = (QI + 7) / 8;   // tiles per share, rounds of eight
    const int it_lo = s * QI, it_hi = min(it_lo + QI, NI);
    uint16_t *sx = p.Sx + static_cast<size_t>(gk) * 16 * MP;
    u64 *flag = p.flags + static_cast<size_t>(gk) * kCtrStride;
    auto load_tile = [&](int it, u32x4 (&dst)[4]) {
        const int u = it / T, jt = it - u * T;
        const char *tile = kc_base + (static_cast<size_t>(u) * m + 16 * jt) * (D * 2);      // scalar
        const int left = m - 1 - 16 * jt;               // last valid row of the tile (may be negative: row m - 1 then)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            dst[i] = *reinterpret_cast<const u32x4 *>(tile + static_cast<ptrdiff_t>(min(4 * i + krow, left)) * 256 + kpc * 16);
    };
    // a key tile in registers -> LDS tile -> the four operands of this lane
    const uint32_t kst = static_cast<uint32_t>(krow * 256 + (kpc ^ krow) * 16);   // piece ^ row, row = 4 i + krow
    auto key_operands = [&](const u32x4 (&src)[4], u32x4 (&dst)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i)     // (kpc ^ (4 i + krow)) = ((kpc ^ krow) with bits 2..3 flipped by i)
            *reinterpret_cast<u32x4 *>(sTile + (kst ^ static_cast<uint32_t>(i * 64)) + 1024 * i) = src[i];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            dst[ks] = *reinterpret_cast<const u32x4 *>(sTile + r16 * 256 + (((4 * ks + kg) ^ r16) & 15) * 16);
    };
    // the scores of one tile (unscaled: sigma multiplies the logits), rows j >= m zero, to the exchange buffer
    auto score_tile = [&](const u32x4 (&src)[4], int it, bool live) {
        u32x4 ka[4];
        key_operands(src, ka);
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ka[ks]), as_bf16x8(qf[ks]), acc, 0, 0, 0);
        const int u = it / T, jt = it - u * T;
        const int j = 16 * jt + 4 * kg;
        uint32_t w[2];
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
            const uint32_t lo = (j + e < m) ? f32_to_bf16_bits(acc[e]) : 0u;
            const uint32_t hi = (j + e + 1 < m) ? f32_to_bf16_bits(acc[e + 1]) : 0u;
            w[e >> 1] = lo | (hi << 16);
        }
        if (r16 < G && live) *reinterpret_cast<u32x2 *>(sx + (u * G + r16) * MP + j) = u32x2_mk(w[0], w[1]);
    };
    u32x4 kf[NRQ][4];
#pragma unroll
    for (int r = 0; r < NRQ; ++r) load_tile(min(it_lo + wave + 8 * r, it_hi - 1), kf[r]);
    if (threadIdx.x == 0) ctr_claim(flag, p.epoch);
    // packed theta: blocks of 8 rows j, each [n][8]; lane (position, kg) of k-step ks reads 16 bytes of block 4 ks + kg
    const char *th_base = reinterpret_cast<const char *>(thp + static_cast<size_t>(h) * m * n);
    uint32_t th_off[NPW];
    LastStep th_last[NPW];
#pragma unroll
    for (int i = 0; i < NPW; ++i) {
        const int pos = p0 + 16 * min(wave + 8 * i, NPT - 1) + r16;
        th_off[i] = static_cast<uint32_t>((kg * n + pos) * 16);
        th_last[i] = last_step(m, n, pos, kg, KS);
    }
    u32x4 lf[KS][NPW];
    auto load_th = [&](int ks) {
        const char *blk = th_base + static_cast<size_t>(ks) * 64 * n;      // scalar
#pragma unroll
        for (int i = 0; i < NPW; ++i)
            lf[ks][i] = *reinterpret_cast<const u32x4_a4 *>(ks < KS - 1 ? blk + th_off[i] : th_base + th_last[i].off);
    };

    // rows r >= RU of the score tile feed the matrix cores too: zeros
    if constexpr (RU < 16) {
        for (int idx = threadIdx.x; idx < (16 - RU) * (LDS / 2); idx += 512)
            reinterpret_cast<uint32_t *>(sS + RU * LDS)[idx] = 0u;
    }

    // this workgroup's share of the scores, out to the L2; once every wave's stores are acknowledged the
    // group's counter moves
#pragma unroll
    for (int r = 0; r < NRQ; ++r) score_tile(kf[r], min(it_lo + wave + 8 * r, it_hi - 1), it_lo + wave + 8 * r < it_hi);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // theta for step 2 is requested now and arrives while the text rows are done and the siblings finish
#pragma unroll
    for (int ks = 0; ks < PDL; ++ks) load_th(ks);
    __shared__ int sAlone;
    lds_barrier();
    if (threadIdx.x == 0) __hip_atomic_fetch_add(flag, static_cast<u64>(1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    TS(4, 7);
    // One word per 128-byte line of this workgroup's quarter of its image blocks' compressed values: memory
    // delivers them into the L2 while steps 1 to 3 run, and step 4 then reads all of them at the L2's latency
    // (requested by all four workgroups at once in step 4, every one of them would wait memory's latency for
    // every line).
    uint32_t touch, touch_u;
    {
        int zero;                                  // (keeps the load, which is from a read-only argument, behind the wait above)
        asm volatile("s_mov_b32 %0, 0" : "=s"(zero)::"memory");
        const size_t vbytes = static_cast<size_t>(UP) * m * D * 2;
        const char *vb = reinterpret_cast<const char *>(Vc + (static_cast<size_t>(bh) * p.I + i0) * m * D);
        touch = *reinterpret_cast<const uint32_t *>(vb + zero + min((static_cast<size_t>(s) * 512 + threadIdx.x) * 128, vbytes - 128));
        // and of this workgroup's eighth of the slice of U (the head's other groups on this XCD read the same slice):
        // PS / 64 of the slice's PS / 8 blocks of m 16-byte rows
        const size_t ubytes = static_cast<size_t>(PS / 64) * m * 16;
        const char *ub = reinterpret_cast<const char *>(Up + static_cast<size_t>(h) * m * n) + (static_cast<size_t>(p0 / 8 + (gl & 7) * (PS / 64)) * m) * 16;
        touch_u = *reinterpret_cast<const uint32_t *>(ub + zero + min(static_cast<size_t>(threadIdx.x & 255) * 128, max(ubytes, static_cast<size_t>(128)) - 128));
    }

    // ---- the text rows of this workgroup's share, completely, while the compressed keys are on their way:
    // logits, weights relative to the share's own maximum per head, and the weighted sum of the value rows
    // (per wavefront: its 2 TT rows, two channels per lane, plain arithmetic)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (xk0 + 4 * i + krow == t_new) tk[i] = tkn;
        u32x4 ka[4];
        key_operands(tk, ka);
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ka[ks]), as_bf16x8(qf[ks]), acc, 0, 0, 0);
        if (wave < TT) {
            f32x4 tl;
#pragma unroll
            for (int e = 0; e < 4; ++e) tl[e] = (x0 + 16 * wave + 4 * kg + e < t) ? acc[e] * p.scale : -INFINITY;
            *reinterpret_cast<f32x4 *>(sTL + r16 * kLTL + 16 * wave + 4 * kg) = tl;
        }
    }
    lds_barrier();
    if (threadIdx.x < 16 * G) {
        const int g = threadIdx.x >> 4, part = threadIdx.x & 15;
        float mxt = -INFINITY;
        for (int xl = part; xl < TR; xl += 16) mxt = fmaxf(mxt, sTL[g * kLTL + xl]);
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) mxt = fmaxf(mxt, __shfl_xor(mxt, o, 64));
        const float mref = mxt == -INFINITY ? 0.f : mxt;       // no row at all: every weight zero, no inf - inf
        float ts = 0.f;
        for (int xl = part; xl < TR; xl += 16) {
            const float pt = __expf(sTL[g * kLTL + xl] - mref);
            sTL[g * kLTL + xl] = pt;
            ts += pt;
        }
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) ts += __shfl_xor(ts, o, 64);
        if (part == 0) { sTm[g] = mxt; sTm[16 + g] = ts; }
    }
    lds_barrier();
    {
        float yt[G][2];
#pragma unroll
        for (int g = 0; g < G; ++g) yt[g][0] = yt[g][1] = 0.f;
        const float *pl = sTL + 2 * TT * wave;
#pragma unroll
        for (int rr = 0; rr < 2 * kTT; rr += 2)
            if (rr < 2 * TT) {          // wave-uniform: arithmetic only, the rows were requested at the top
                // (rows beyond the sequence's own are clamped copies with weight zero; in a ragged batch they may be
                // anything, so they are selected away rather than multiplied)
                const uint32_t va = xv0 + rr == t_new ? tvn : (!RAG || xv0 + rr < t) ? tv[rr] : 0u;
                const uint32_t vc = xv0 + rr + 1 == t_new ? tvn : (!RAG || xv0 + rr + 1 < t) ? tv[rr + 1] : 0u;
                const float a0 = bf_lo(va), a1 = bf_hi(va), c0 = bf_lo(vc), c1 = bf_hi(vc);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const f32x2 pp = *reinterpret_cast<const f32x2 *>(pl + g * kLTL + rr);
                    yt[g][0] = fmaf(pp.y, c0, fmaf(pp.x, a0, yt[g][0]));
                    yt[g][1] = fmaf(pp.y, c1, fmaf(pp.x, a1, yt[g][1]));
                }
            }
#pragma unroll
        for (int g = 0; g < G; ++g)
            *reinterpret_cast<f32x2 *>(sYt + (wave * 8 + g) * D + 2 * lane) = f32x2_mk(yt[g][0], yt[g][1]);
    }
    TS(4, 6);
    // all shares of the scores there?  (waiting is bounded: siblings that are not resident, or a counter word that
    // holds something else, end in this workgroup computing every share itself -- slower, same result)
    if (threadIdx.x == 0) {
        const u64 want = ctr_word(p.epoch, static_cast<unsigned>(p.F));
        const unsigned long long t0 = wall_clock64();
        bool all = false;
        if (p.wait_ticks > 0) {
            do {
                for (int k = 0; k < 8 && !all; ++k) {            // the clock is read once per 8 polls
                    const u64 v = ctr_peek(flag);
                    all = v >= want && static_cast<unsigned>(v >> 32) == p.epoch;
                }
            } while (!all && wall_clock64() - t0 < static_cast<unsigned long long>(p.wait_ticks));
        }
        sAlone = all ? 0 : 1;
        if (!all && p.fallbacks) atomicAdd(p.fallbacks, 1u);
    }
    lds_barrier();
    if (sAlone) {
#pragma unroll 1
        for (int r = 0; r < NRS; ++r) {
            const int it = wave + 8 * r;
            u32x4 kx[4];
            load_tile(min(it, NI - 1), kx);
            score_tile(kx, min(it, NI - 1), it < NI);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        lds_barrier();
    }
    asm volatile("buffer_inv sc0" ::: "memory");
    // the group's scores -> LDS: RU rows of MP values, 16 bytes per thread and pass
    {
        constexpr int PPR = MP / 8, NPC = RU * PPR, NPS = (NPC + 511) / 512;
        u32x4 sv[NPS];
        int sidx[NPS];
#pragma unroll
        for (int k = 0; k < NPS; ++k) {
            sidx[k] = min(static_cast<int>(threadIdx.x) + 512 * k, NPC - 1);
            const int row = sidx[k] / PPR, c = sidx[k] - row * PPR;
            sv[k] = *reinterpret_cast<const u32x4 *>(sx + row * MP + 8 * c);
        }
#pragma unroll
        for (int k = 0; k < NPS; ++k) {
            const int row = sidx[k] / PPR, c = sidx[k] - row * PPR;
            *reinterpret_cast<u32x4 *>(sS + row * LDS + 8 * c) = sv[k];
        }
    }
    lds_barrier();
    TS(4, 1);


    // ---- step 2: L^T[pos][row] = sum_j theta[j][pos] S[row][j] for this wave's position tiles ----------
    // packed U (kvc_pack_u): blocks of 8 positions, each [m][8]; lane (row j, kg) of k-step ks reads the 16 bytes of
    // block p0 / 8 + 4 ks + kg -- 16 consecutive rows are 256 contiguous bytes, so a quarter-wave reads two whole lines
    // and the registers are MFMA operands as they arrive (like theta's; rows of the plain [m][n] form would have to be
    // loaded whole and turned around through LDS)
    const char *u_base = reinterpret_cast<const char *>(Up + static_cast<size_t>(h) * m * n) + (static_cast<size_t>(p0 / 8 + kg) * m) * 16;
    u32x4 uf[NRW][KP];
    auto u_partial = [](int r) { return 8 * r + 7 >= TI; };
    auto u_tile = [&](int r) { return min(wave + 8 * r, T - 1); };
    auto load_u = [&](int r) {
        const int jt = u_tile(r);
        const uint32_t row = static_cast<uint32_t>(u_partial(r) ? min(16 * jt + r16, m - 1) : 16 * jt + r16) * 16u;
#pragma unroll
        for (int ks = 0; ks < KP; ++ks)
            uf[r][ks] = *reinterpret_cast<const u32x4 *>(u_base + static_cast<size_t>(ks) * 64 * m + row);
    };
    f32x4 accL[NPW];
#pragma unroll
    for (int i = 0; i < NPW; ++i) accL[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        if (ks + PDL < KS) load_th(ks + PDL);
        if (ks == (KS > PDL ? KS - PDL : 0)) {
#pragma unroll
            for (int r = 0; r < PDW; ++r) load_u(r);
        }
        const bf16x8 sfr = *reinterpret_cast<const bf16x8 *>(sS + r16 * LDS + 32 * ks + 8 * kg);
#pragma unroll
        for (int i = 0; i < NPW; ++i) {
            u32x4 a = lf[ks][i];
            if (ks == KS - 1) a = shift_window(a, th_last[i].ds, th_last[i].bs);
            accL[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a), sfr, accL[i], 0, 0, 0);
        }
    }
    // (sigma multiplies the logits here, 8 values per lane, instead of the scores)
#pragma unroll
    for (int i = 0; i < NPW; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) accL[i][e] *= p.scale;
    // slice maximum of row r16: lane, wave, workgroup
    {
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < NPW; ++i)
            if (NPT % 8 == 0 || wave + 8 * i < NPT) {
#pragma unroll
                for (int e = 0; e < 4; ++e) mx = fmaxf(mx, accL[i][e]);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        if (kg == 0) sRed[r16 * 8 + wave] = mx;
    }
    lds_barrier();
    TS(4, 2);
    auto row_max = [&](int r) {
        const f32x4 a = *reinterpret_cast<const f32x4 *>(sRed + r * 8), c = *reinterpret_cast<const f32x4 *>(sRed + r * 8 + 4);
        return fmaxf(fmaxf(fmaxf(a[0], a[1]), fmaxf(a[2], a[3])), fmaxf(fmaxf(c[0], c[1]), fmaxf(c[2], c[3])));
    };
    {
        const float mx = row_max(r16);
        float sm = 0.f;
#pragma unroll
        for (int i = 0; i < NPW; ++i) {
            const uint32_t a0 = f32_to_bf16_bits(__expf(accL[i][0] - mx)), a1 = f32_to_bf16_bits(__expf(accL[i][1] - mx));
            const uint32_t a2 = f32_to_bf16_bits(__expf(accL[i][2] - mx)), a3 = f32_to_bf16_bits(__expf(accL[i][3] - mx));
            if (NPT % 8 == 0 || wave + 8 * i < NPT) {
                sm += __uint_as_float(a0 << 16) + __uint_as_float(a1 << 16) + __uint_as_float(a2 << 16) + __uint_as_float(a3 << 16);
                *reinterpret_cast<u32x2 *>(sP + r16 * LDP + 16 * (wave + 8 * i) + 4 * kg) = u32x2_mk(a0 | (a1 << 16), a2 | (a3 << 16));
            }
        }
        sm += __shfl_xor(sm, 16, 64);
        sm += __shfl_xor(sm, 32, 64);
        if (kg == 0) sRed[128 + r16 * 8 + wave] = sm;
    }
    lds_barrier();
    TS(4, 3);

    asm volatile("" ::"v"(touch), "v"(touch_u));
    // ---- step 3: W^T[j][row] = sum_pos U[j][pos] P[row][pos] for this wave's tiles of 16 rows of U ------
    const char *vc_base = reinterpret_cast<const char *>(Vc + (static_cast<size_t>(bh) * p.I + i0) * m * D);
    const int cch = 16 * wave + r16;                     // this lane's channel in step 4
    const uint32_t vc_off = static_cast<uint32_t>((kg * D + cch) * 16);
    const LastStep vc_last = last_step(m, D, cch, kg, KS);
    u32x4 vf[KS][UP];
    auto load_v = [&](int ks) {
#pragma unroll
        for (int u = 0; u < UP; ++u) {
            const char *blk = vc_base + static_cast<size_t>(u) * m * (D * 2) + (ks < KS - 1 ? ks * (64 * D) : 0);   // scalar
            vf[ks][u] = *reinterpret_cast<const u32x4_a4 *>(blk + (ks < KS - 1 ? vc_off : vc_last.off));
        }
    };
    bf16x8 pfr[KP];
#pragma unroll
    for (int ks = 0; ks < KP; ++ks) pfr[ks] = *reinterpret_cast<const bf16x8 *>(sP + r16 * LDP + 32 * ks + 8 * kg);
#pragma unroll
    for (int r = 0; r < NRW; ++r) {
        if (r + PDW < NRW) load_u(r + PDW);
        if (r + PDW == NRW) {
#pragma unroll
            for (int ks = 0; ks < PDY; ++ks) load_v(ks);
        }
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KP; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(uf[r][ks]), pfr[ks], acc, 0, 0, 0);
        const int jt = wave + 8 * r;
        const int j = 16 * u_tile(r) + 4 * kg;
        uint32_t w0, w1;
        if (!u_partial(r)) {
            w0 = f32_to_bf16_bits(acc[0]) | (static_cast<uint32_t>(f32_to_bf16_bits(acc[1])) << 16);
            w1 = f32_to_bf16_bits(acc[2]) | (static_cast<uint32_t>(f32_to_bf16_bits(acc[3])) << 16);
        } else {
            const uint32_t b0 = (j + 0 < m) ? f32_to_bf16_bits(acc[0]) : 0u, b1 = (j + 1 < m) ? f32_to_bf16_bits(acc[1]) : 0u;
            const uint32_t b2 = (j + 2 < m) ? f32_to_bf16_bits(acc[2]) : 0u, b3 = (j + 3 < m) ? f32_to_bf16_bits(acc[3]) : 0u;
            w0 = b0 | (b1 << 16);
            w1 = b2 | (b3 << 16);
        }
        if (8 * r + 7 < T || jt < T) *reinterpret_cast<u32x2 *>(sW + r16 * LDS + j) = u32x2_mk(w0, w1);
    }
    lds_barrier();
    TS(4, 4);

    // ---- step 4: Y^T[c][row] = sum_j Vc^T[c][j] W[row][j], per image block; wave w owns channels 16 w ... ----
    f32x4 o[UP];
#pragma unroll
    for (int u = 0; u < UP; ++u) o[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        if (ks + PDY < KS) load_v(ks + PDY);
        const bf16x8 wfr = *reinterpret_cast<const bf16x8 *>(sW + r16 * LDS + 32 * ks + 8 * kg);
#pragma unroll
        for (int u = 0; u < UP; ++u) {
            u32x4 a = vf[ks][u];
            if (ks == KS - 1) a = shift_window(a, vc_last.ds, vc_last.bs);
            o[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a), wfr, o[u], 0, 0, 0);
        }
    }
    // the image blocks' outputs, brought to the head's joint maximum and summed into one record
    auto row_sum = [&](int r) {
        const f32x4 a = *reinterpret_cast<const f32x4 *>(sRed + 128 + r * 8), c = *reinterpret_cast<const f32x4 *>(sRed + 128 + r * 8 + 4);
        return ((a[0] + a[1]) + (a[2] + a[3])) + ((c[0] + c[1]) + (c[2] + c[3]));
    };
    const int un_mine = r16 / G, g_mine = min(r16 - un_mine * G, G - 1);
    float rmx[UP];
    // joint maximum of this lane's query head over the workgroup's image blocks and text rows.  An image block
    // the sequence does not have (ragged batch) takes no part: whatever its capsule slot holds went through the
    // products above in rows and blocks of its own, which are selected away here (never multiplied by zero:
    // the slot may hold NaNs)
    float gm = sTm[g_mine];
#pragma unroll
    for (int u = 0; u < UP; ++u) {
        rmx[u] = (!RAG || i0 + u < n_img) ? row_max(u * G + g_mine) : -INFINITY;
        gm = fmaxf(gm, rmx[u]);
    }
    if constexpr (RAG) gm = gm == -INFINITY ? 0.f : gm;       // nothing at all in this workgroup: a record without mass
    f32x4 ysum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < UP; ++u) {
        const bool mine = un_mine == u && r16 < RU && (!RAG || i0 + u < n_img);        // rows of other blocks: cross terms
        const float sc = __expf(rmx[u] - gm);
#pragma unroll
        for (int e = 0; e < 4; ++e) ysum[e] += mine ? sc * o[u][e] : 0.f;
    }
    if constexpr (UP > 1) {
        if constexpr ((G & (G - 1)) == 0) {
#pragma unroll
            for (int o2 = G; o2 < 16; o2 <<= 1)
#pragma unroll
                for (int e = 0; e < 4; ++e) ysum[e] += __shfl_xor(ysum[e], o2, 64);
        } else {
            static_assert(UP <= 2, "blocks of a tile are summed with one exchange");
#pragma unroll
            for (int e = 0; e < 4; ++e) ysum[e] += __shfl(ysum[e], (lane & 48) | ((r16 + G) & 15), 64);
        }
    }
    if (r16 < G) {
        float *yp = p.Ypart + (static_cast<size_t>(bh) * p.nparts + pi) * p.rec;
        f32x4 yt = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w8 = 0; w8 < 8; ++w8) {
            const f32x4 part = *reinterpret_cast<const f32x4 *>(sYt + (w8 * 8 + r16) * D + 16 * wave + 4 * kg);
            yt[0] += part[0]; yt[1] += part[1]; yt[2] += part[2]; yt[3] += part[3];
        }
        const float tsc = __expf(sTm[r16] - gm);             // the text share's own maximum -> the joint one (exp(-inf) = 0 without rows)
        *reinterpret_cast<f32x4 *>(yp + r16 * D + 16 * wave + 4 * kg) =
            f32x4_mk(ysum[0] + tsc * yt[0], ysum[1] + tsc * yt[1], ysum[2] + tsc * yt[2], ysum[3] + tsc * yt[3]);
        if (wave == 0 && kg == 0) {
            float vs = 0.f;
#pragma unroll
            for (int u = 0; u < UP; ++u) vs += (!RAG || i0 + u < n_img) ? row_sum(u * G + r16) * __expf(rmx[u] - gm) : 0.f;
            yp[G * D + r16] = (RAG && vs + tsc * sTm[16 + r16] == 0.f) ? -INFINITY : gm;
            yp[G * D + G + r16] = vs + tsc * sTm[16 + r16];
            yp[G * D + 2 * G + r16] = vs;
        }
    }
    // Sec. 3.2: the text cache keeps growing as in the backbone -- store the new token's k, v
    if (fresh && t_in >= x0 && t_in < x0 + TR && threadIdx.x < 32) {
        const int half = threadIdx.x >> 4, piece = threadIdx.x & 15;
        const uint16_t *src = (half ? v_new : k_new) + static_cast<size_t>(bh) * D;
        uint16_t *dst = (half ? Vt : Kt) + (static_cast<size_t>(bh) * p.cap + t_in) * D;
        *(reinterpret_cast<u32x4 *>(dst) + piece) = *(reinterpret_cast<const u32x4 *>(src) + piece);
    }
    TS(4, 5);
}

// Joint softmax over the part records of one (batch element, query head): as fd_finalize_few of the
// four-kernel form, with the vision share of each part's sum carried in the record (a part holds image
// blocks and text rows together); `+ (sum P_vis) mu` per Sec. 3.1 (values are stored centred).
template <int PB>
__global__ __launch_bounds__(128) void fs_finalize(const float *__restrict__ Ypart, const uint16_t *__restrict__ mu,
                                                   uint16_t *__restrict__ out, float *__restrict__ lse, int Hkv,
                                                   unsigned qHkv, int G, unsigned qG, int np, int rec, int Hq,
                                                   u64 *flags, int nflags)
{
    const int bgi = quot(blockIdx.x, qHkv), h = blockIdx.x - bgi * Hkv;
    const int b = quot(bgi, qG), g = bgi - b * G;
    const int bg = b * Hq + h * G + g;
    const int lane = threadIdx.x & 63, c = threadIdx.x;
    const int GD = G * D;
    const float *yb = Ypart + static_cast<size_t>(b * Hkv + h) * np * rec;
    const int pl = min(lane, np - 1);
    float ml = yb[static_cast<size_t>(pl) * rec + GD + g];
    float sl = yb[static_cast<size_t>(pl) * rec + GD + G + g];
    float vl = yb[static_cast<size_t>(pl) * rec + GD + 2 * G + g];
    __builtin_amdgcn_sched_barrier(0);
    const float *yc = yb + g * D + c;
    float v[PB];
#pragma unroll
    for (int k = 0; k < PB; ++k) v[k] = yc[static_cast<size_t>(min(k, np - 1)) * rec];
    const uint16_t mub = mu[static_cast<size_t>(h) * D + c];
    __builtin_amdgcn_sched_barrier(0);
    if (lane >= np) { ml = -INFINITY; sl = 0.f; vl = 0.f; }
    const float mx = wave_max(ml);
    const float a = __expf(ml - mx);
    const float z = wave_sum(sl * a);
    const float zv = wave_sum(vl * a);
    const float rz = 1.f / z;
    const float wgt = a * rz;
    float y = (zv * rz) * bf_lo(mub);
#pragma unroll
    for (int k = 0; k < PB; ++k) y += __shfl(wgt, k, 64) * v[k];
    out[static_cast<size_t>(bg) * D + c] = f32_to_bf16_bits(y);
    if (c == 0 && lse) lse[bg] = mx + __logf(z);
    // the arrival counters of fs_stream go back to zero
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < nflags; i += 128) flags[static_cast<size_t>(i) * kCtrStride] = 0ull;
}

int stream_up(int G) { return G == 1 ? 16 : G == 2 ? 8 : G == 4 ? 4 : (G >= 6 && G <= 8) ? 2 : 0; }

// the slice of positions a workgroup takes for an image block of n positions (0: no instance)
int stream_ps(int n) { return n == 1024 ? 256 : 0; }

bool make_splan(SPlan &p, const DecodeCall &c, void *base, size_t *bytes)
{
    const kvc_shape &s = c.s;
    p.B = s.batch; p.Hq = s.n_q_heads; p.Hkv = s.n_kv_heads;
    p.I = s.n_images; p.n = s.n_img_tokens; p.m = s.m;
    p.t = c.t; p.t_in = c.t_in; p.cap = c.cap; p.scale = c.scale;
    const int G = p.Hq / p.Hkv, UP = stream_up(G), PS = stream_ps(p.n);
    if (!UP || !PS || p.I < 1 || p.I % UP) return false;
    p.IU = p.I / UP;
    p.F = p.n / PS;
    p.NGR = p.Hkv * p.B * p.IU;
    p.chunk = (p.NGR + 7) / 8;
    p.nparts = p.IU * p.F;
    if (p.nparts > 64) return false;
    const int per = (p.t + p.nparts - 1) / p.nparts;
    p.TT = (per + 15) / 16;
    if (p.TT > kTT) return false;
    p.rec = static_cast<int>(align_up(G * D + 3 * G, 4));
    p.qF = quot_multiplier(p.F); p.qBIU = quot_multiplier(p.B * p.IU); p.qIU = quot_multiplier(p.IU);
    // quot(): dividends below 2^32 / divisor
    if (static_cast<long>(8) * p.chunk * p.F * std::max(p.F, p.B * p.IU) >= (1l << 31)) return false;
    if (p.F != 4 || p.NGR > kMaxFlags) return false;
    // workspace: arrival counters (the same 64 KB the four-kernel form keeps its counters in), part records, scores
    const size_t fbytes = static_cast<size_t>(kMaxFlags) * kCtrStride * sizeof(u64);
    const size_t ybytes = align_up(static_cast<size_t>(p.B) * p.Hkv * p.nparts * p.rec * sizeof(float), 256);
    const size_t sbytes = static_cast<size_t>(p.NGR) * 16 * (32 * ((p.m + 31) / 32)) * sizeof(uint16_t);
    p.flags = static_cast<u64 *>(base);
    p.Ypart = reinterpret_cast<float *>(static_cast<char *>(base) + fbytes);
    p.Sx = reinterpret_cast<uint16_t *>(static_cast<char *>(base) + fbytes + ybytes);
    p.epoch = 0; p.wait_ticks = 0; p.fallbacks = nullptr;
    p.n_img = c.n_images_dev; p.tlen = c.text_len_dev;
    *bytes = fbytes + ybytes + align_up(sbytes, 256);
    return true;
}

template <int G, int UP, int PS, int KS, bool RAG> bool launch_s2(const SPlan &p, const DecodeCall &c)
{
    constexpr size_t lds = stream_lds_bytes(KS, PS);
    static_assert(lds <= 160 * 1024, "LDS of a compute unit");
    static bool attr_set[kMaxDevices] = {};
    if (!allow_lds(reinterpret_cast<const void *>(fs_stream<G, UP, PS, KS, RAG>), lds, attr_set)) return false;
    // without text rows the (never used) text pointers still have to be addresses that can be read
    uint16_t *Kt = static_cast<uint16_t *>(c.Kt), *Vt = static_cast<uint16_t *>(c.Vt);
    if (p.cap == 0 || !Kt || !Vt) { Kt = Vt = const_cast<uint16_t *>(static_cast<const uint16_t *>(c.q)); }
    fs_stream<G, UP, PS, KS, RAG><<<8 * p.chunk * p.F, 512, lds, c.stream>>>(
        static_cast<const uint16_t *>(c.q), static_cast<const uint16_t *>(c.Kc), static_cast<const uint16_t *>(c.theta_packed),
        static_cast<const uint16_t *>(c.U_packed), static_cast<const uint16_t *>(c.Vc), Kt, Vt,
        static_cast<const uint16_t *>(c.k_new), static_cast<const uint16_t *>(c.v_new), p);
    return true;
}

template <int G, int UP, int PS, int KS> bool launch_s(const SPlan &p, const DecodeCall &c)
{
    return p.n_img ? launch_s2<G, UP, PS, KS, true>(p, c) : launch_s2<G, UP, PS, KS, false>(p, c);
}

// instances: (group size, compressed length in 32-row steps)
template <int G, int UP> int launch_for_ks(const SPlan &p, const DecodeCall &c, int KS, bool probe)
{
    switch (KS) {
#define KVC_STREAM_CASE(K) case K: return probe ? 1 : (launch_s<G, UP, 256, K>(p, c) ? 1 : -1);
    // every compressed length of n = 1024
    KVC_STREAM_CASE(1) KVC_STREAM_CASE(2) KVC_STREAM_CASE(3) KVC_STREAM_CASE(4) KVC_STREAM_CASE(5) KVC_STREAM_CASE(6)
    KVC_STREAM_CASE(7) KVC_STREAM_CASE(8) KVC_STREAM_CASE(9) KVC_STREAM_CASE(10) KVC_STREAM_CASE(11) KVC_STREAM_CASE(12)
    KVC_STREAM_CASE(13) KVC_STREAM_CASE(14) KVC_STREAM_CASE(15) KVC_STREAM_CASE(16) KVC_STREAM_CASE(17) KVC_STREAM_CASE(18)
    KVC_STREAM_CASE(19) KVC_STREAM_CASE(20) KVC_STREAM_CASE(21) KVC_STREAM_CASE(22) KVC_STREAM_CASE(23) KVC_STREAM_CASE(24)
    KVC_STREAM_CASE(25) KVC_STREAM_CASE(26) KVC_STREAM_CASE(27) KVC_STREAM_CASE(28) KVC_STREAM_CASE(29) KVC_STREAM_CASE(30)
    KVC_STREAM_CASE(31) KVC_STREAM_CASE(32)
#undef KVC_STREAM_CASE
    default: return 0;
    }
}

// 1: launched (or, probing, an instance exists); 0: no instance; -1: launch failed
int launch_stream(const SPlan &p, const DecodeCall &c, bool probe)
{
    const int G = p.Hq / p.Hkv, KS = (p.m + 31) / 32;
    switch (G) {
    case 4: return launch_for_ks<4, 4>(p, c, KS, probe);
    case 6: return launch_for_ks<6, 2>(p, c, KS, probe);
    case 7: return launch_for_ks<7, 2>(p, c, KS, probe);
    case 8: return launch_for_ks<8, 2>(p, c, KS, probe);
    default: return 0;
    }
}

template <int PB> void launch_fin(const SPlan &p, const DecodeCall &c)
{
    const int G = p.Hq / p.Hkv;
    fs_finalize<PB><<<p.B * p.Hq, 128, 0, c.stream>>>(p.Ypart, static_cast<const uint16_t *>(c.mu), static_cast<uint16_t *>(c.out),
                                                      c.lse, p.Hkv, quot_multiplier(p.Hkv), G, quot_multiplier(G), p.nparts,
                                                      p.rec, p.Hq, p.flags, p.NGR);
}

}  // namespace

void stream_decode_knob(int mode) { g_stream_mode = mode; }
long stream_decode_calls() { return g_stream_calls.load(); }

size_t stream_decode_ws_bytes(const kvc_shape &s, int32_t max_text)
{
    // (the text length only decides whether a call is taken, not the size)
    DecodeCall c;
    c.s = s; c.t = c.t_in = 0; c.cap = max_text; c.scale = 1.f;
    SPlan p;
    size_t bytes = 0;
    return make_splan(p, c, nullptr, &bytes) ? bytes : 0;
}

// true: the call was taken (status in *st); false: not this path's shape, nothing was launched
bool stream_decode(const DecodeCall &c, kvc_status *st)
{
    if (g_stream_mode == 0 || !c.theta_packed || !c.U_packed || c.static_variant) return false;
    if ((c.n_images_dev == nullptr) != (c.text_len_dev == nullptr)) return false;
    if (c.s.dtype != KVC_BF16 || c.s.head_dim != D) return false;
    SPlan p;
    size_t bytes = 0;
    if (!make_splan(p, c, c.ws, &bytes)) return false;
    if (launch_stream(p, c, true) != 1) return false;
    if (g_stream_mode < 0) {
        // built-in rule: calls small enough that launches and hand-overs, not bytes, decide the time of the
        // four-kernel form: fewer than two workgroups per compute unit (at two, B = 8 of the headline model's
        // shape, the two forms take the same time: 36.3 against 35.7 us per call; at B = 2, 18.8 against 20.7)
        if (8 * p.chunk * p.F >= 512) return false;
    }
    if (bytes > c.ws_bytes) { *st = KVC_ERR_WORKSPACE; return true; }
    p.epoch = next_decode_epoch();
    p.wait_ticks = decode_wait_ticks();
    p.fallbacks = decode_fallback_counter();
#if defined(KVC_TIMELINE)
    p.tl = c.ws_bytes >= bytes + kTimelineBytes
               ? reinterpret_cast<unsigned long long *>(static_cast<char *>(c.ws) + ((c.ws_bytes - kTimelineBytes) & ~size_t(255)))
               : nullptr;
#endif
    if (launch_stream(p, c, false) != 1) { *st = KVC_ERR_HIP; return true; }
    ++g_stream_calls;
    switch ((p.nparts + 7) >> 3) {
    case 1: launch_fin<8>(p, c); break;
    case 2: launch_fin<16>(p, c); break;
    case 3: launch_fin<24>(p, c); break;
    case 4: launch_fin<32>(p, c); break;
    case 5: launch_fin<40>(p, c); break;
    case 6: launch_fin<48>(p, c); break;
    case 7: launch_fin<56>(p, c); break;
    default: launch_fin<64>(p, c); break;
    }
    *st = hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_HIP;
    return true;
}

// ---- packed form of theta ------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(256) void pack_theta_kernel(const T *__restrict__ theta, T *__restrict__ packed, int m, int n)
{
    const T *src = theta + static_cast<size_t>(blockIdx.y) * m * n;
    T *dst = packed + static_cast<size_t>(blockIdx.y) * m * n;
    const int j = blockIdx.x;
    for (int pos = threadIdx.x; pos < n; pos += 256) dst[vc_offset(j, pos, m, n)] = src[static_cast<size_t>(j) * n + pos];
}

// U -> blocks of 8 positions, each [m][8]: element (row j, position pos) at vc_offset(pos, j, n, m)
template <class T>
__global__ __launch_bounds__(256) void pack_u_kernel(const T *__restrict__ U, T *__restrict__ packed, int m, int n)
{
    const T *src = U + static_cast<size_t>(blockIdx.y) * m * n;
    T *dst = packed + static_cast<size_t>(blockIdx.y) * m * n;
    const int j = blockIdx.x;
    for (int pos = threadIdx.x; pos < n; pos += 256) dst[vc_offset(pos, j, n, m)] = src[static_cast<size_t>(j) * n + pos];
}

kvc_status pack_u(const kvc_shape &s, const void *U, void *packed, hipStream_t stream)
{
    const dim3 grid(s.m, s.n_kv_heads);
    if (s.dtype == KVC_F32)
        pack_u_kernel<float><<<grid, 256, 0, stream>>>(static_cast<const float *>(U), static_cast<float *>(packed), s.m, s.n_img_tokens);
    else
        pack_u_kernel<uint16_t><<<grid, 256, 0, stream>>>(static_cast<const uint16_t *>(U), static_cast<uint16_t *>(packed), s.m, s.n_img_tokens);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_HIP;
}

kvc_status pack_theta(const kvc_shape &s, const void *theta, void *packed, hipStream_t stream)
{
    const dim3 grid(s.m, s.n_kv_heads);
    if (s.dtype == KVC_F32)
        pack_theta_kernel<float><<<grid, 256, 0, stream>>>(static_cast<const float *>(theta), static_cast<float *>(packed), s.m, s.n_img_tokens);
    else
        pack_theta_kernel<uint16_t><<<grid, 256, 0, stream>>>(static_cast<const uint16_t *>(theta), static_cast<uint16_t *>(packed), s.m, s.n_img_tokens);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_HIP;
}

}  // namespace kvc
