// Matrix-core decode path of KVCapsule for gfx950: bf16 storage, head_dim 128.
//
// One decode step of one layer = four launches (three where the first two run as one, fab_fused)
// that follow Alg. 1 of the paper
// (score-space order), with the softmax taken jointly over vision and text keys
// (Sec. 3.2) by carrying (max, sum) statistics per part and merging them at the end:
//
//   fa_scores   streams the compressed keys Kc from HBM once: S = sigma q Kc^T (Alg. 1 step 1),
//               one 16x16x32 MFMA tile per 16 key rows.
//   text_part   (a device function, run by extra workgroups of fc_fused) handles 128 rows of the
//               text cache completely: logits, exp relative to the chunk's own maximum,
//               P V_text (V_text transposed through LDS), and writes a finished part record; the
//               chunk that owns row text_len also stores the new token's k, v (Sec. 3.2: text KV
//               is kept as it is).
//   fb_probs    L = S theta (step 2) as a skinny GEMM per KV head, 64 (or 128) query rows x 64
//               positions per workgroup with the theta chunk transposed into LDS on the way
//               in; emits P = exp(L - tile max) in bf16 and the tile's (max, sum) per row.
//   fc_fused    per (KV head, group of up to 32 query rows = whole image blocks, 64 rows j
//               of the capsule): W = sum_tiles alpha_tile (P_tile U_tile^T) with
//               alpha = exp(tile max - block max) (step 3), then out_part = W Vc over the same
//               64 rows of the compressed values (step 4; Vc's blocked layout is the MFMA
//               operand), un-normalised, with the block's (max, sum).
//   fd_finalize_few / fd_finalize  merge the parts of each (batch, query head) with the joint
//               softmax statistics, add (sum P_vis) mu, write out and lse.
//
// Only S and P (bf16), the tile statistics and the part records cross kernel boundaries;
// K_hat, V_hat and W never exist in memory.
//
// What the measurements on this chip dictate:
//  * kernel boundaries are the only grid-wide synchronisation: a device-scope fence inside a
//    kernel writes back and invalidates an XCD's whole L2 and costs far more than a launch
//    (fab_fused synchronises the workgroups of one XCD only, through its L2, without fences);
//  * a load whose lanes use only half of each 128-byte line (what an MFMA operand fetched
//    straight from a row-major matrix does: 16 rows x 64 bytes) runs at half the L1 rate; for U
//    in fc_fused, which is bound by L2 bandwidth, that measured equal to staging coalesced loads
//    through LDS, so the simpler direct operand loads are used;
//  * loads are requested in the order the matrix work needs them, the bulk (second half of U,
//    compressed values) only after the first MFMAs are under way: requesting everything up front
//    stalls the instruction stream on a full memory queue before any matrix work starts;
//  * loops that feed MFMAs carry no tests (trip counts are template parameters): a guarded loop
//    makes the compiler move accumulators between register files at every step;
//  * MFMA results are stored directly (no cross-lane reductions beyond two steps) and code stays
//    small (cold instruction cache per launch);
//  * what stands in front of a kernel's first load is paid by every workgroup: the values it takes
//    are plain leading kernel arguments, which the hardware hands to a wave in registers (kernel-
//    argument preload, up to 14 dwords; the rest of the plan is fetched from memory behind the first
//    loads), and indices are divided by multiplication (quot).
//
// Query rows of one KV head: image block ub = b*I + i owns G consecutive rows (one per query head of
// the group), and UPB = 2^UPBs whole image blocks fill a 64-row block (the rest of its rows unused), so
// that consecutive image blocks share MFMA tiles and no image block straddles two 64-row blocks.
#include "kvc_decode_dev.h"

#include <algorithm>
#include <atomic>
#include <mutex>

namespace kvc {
namespace {

using namespace dd;

// developer knobs (kvc_dev_decode_knobs) and the call counter that numbers fab_fused's epochs
std::atomic<unsigned> g_epoch{0};
int g_wait_ticks = 2000;          // 20 us: a few launch latencies; a workgroup that waits longer computes alone
int g_force_nt = 0;               // row tiles per fc_fused workgroup (0: rule in make_plan_layout)
int g_use_packed_u = 1;           // developer switch: 0 reads the plain U even where the packed form is given
int g_separate = 0;               // 1: fa_scores and fb_probs as separate launches

// ------------------------------------------------------------------------------------------
// fa_scores: Alg. 1 step 1 on the compressed keys (vision workgroups), and the complete
// attention part of 128 text rows (text workgroups).
// MFMA tile: A = 16 key rows x 32 channels, B = 32 channels x 16 query heads of the group,
// D[key row][head]; a lane ends up with 4 consecutive key rows of one head.
// Part record in Ypart: [G][D] floats of un-normalised output, [G] maxima, [G] sums.
// ------------------------------------------------------------------------------------------
// (leading arguments: what stands in front of the first loads, preloaded into registers, see fb_probs)
template <int G, bool TEXT, bool RAG>
__global__ __launch_bounds__(256) void fa_scores(const uint16_t *__restrict__ q, const uint16_t *__restrict__ Kc,
                                                 int a_vis_tiles, unsigned a_qTPU, int a_tiles_per_unit, unsigned a_qI,
                                                 int a_I, unsigned a_qHkv, int a_Hkv, int a_m, int a_Hq, int a_ntext_a,
                                                 Plan p, uint16_t *__restrict__ Kt, uint16_t *__restrict__ Vt,
                                                 const uint16_t *__restrict__ k_new,
                                                 const uint16_t *__restrict__ v_new)
{
    p.vis_tiles = a_vis_tiles; p.qTPU = a_qTPU; p.tiles_per_unit = a_tiles_per_unit; p.qI = a_qI; p.I = a_I;
    p.qHkv = a_qHkv; p.Hkv = a_Hkv; p.m = a_m; p.Hq = a_Hq; p.ntext_a = a_ntext_a;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, kg = lane >> 4;
    TS(0, 0);

    // without vision tokens there is no fc_fused launch: the text chunks are handled here (TEXT; the
    // instance for the usual case reserves no LDS)
    if constexpr (TEXT) {
        if (static_cast<int>(blockIdx.x) < p.ntext_a) {
            __shared__ __align__(16) uint16_t sText[kTextLds / 2];
            text_part<G, RAG>(p, q, Kt, Vt, k_new, v_new, sText, blockIdx.x, threadIdx.x, true);
            return;
        }
    }

    // ---------------- vision: kTPW tiles of 16 compressed key rows per wave ----------------
    const int tile0 = ((blockIdx.x - p.ntext_a) * 4 + wave) * kTPW;
    u32x4 kf[kTPW][4], qf[kTPW][4];
    bool live[kTPW];
    int bh_prev = -1;
#pragma unroll
    for (int tt = 0; tt < kTPW; ++tt) {
        const int tile = tile0 + tt;
        live[tt] = tile < p.vis_tiles;
        if (!live[tt]) continue;
        const int u = quot(tile, p.qTPU), jt = tile - u * p.tiles_per_unit;
        const int bh = quot(u, p.qI);
        const int b = quot(bh, p.qHkv), h = bh - b * p.Hkv;
        const int row = min(jt * 16 + r16, p.m - 1);
        const u32x4 *kp = reinterpret_cast<const u32x4 *>(Kc + (static_cast<size_t>(u) * p.m + row) * D) + kg;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) kf[tt][ks] = kp[4 * ks];
        // tiles of one (batch, KV head) share the query rows: the second tile of a wave reloads them
        // only when it belongs to another one
        if (tt == 0 || bh != bh_prev) {
            const u32x4 *qp = reinterpret_cast<const u32x4 *>(q + (static_cast<size_t>(b) * p.Hq + h * G + min(r16, G - 1)) * D) + kg;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) qf[tt][ks] = qp[4 * ks];
        } else {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) qf[tt][ks] = qf[tt - 1][ks];
        }
        bh_prev = bh;
    }
    fetch_now(p.scale, p.S, p.R_pad, p.m_pad, p.m16);
    TS(0, 1);
#pragma unroll
    for (int tt = 0; tt < kTPW; ++tt) {
        if (!live[tt]) continue;
        const int tile = tile0 + tt;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kf[tt][ks]), as_bf16x8(qf[tt][ks]), acc, 0, 0, 0);
        if (r16 >= G) continue;      // columns beyond the group are copies of head G-1
        const int u = quot(tile, p.qTPU), jt = tile - u * p.tiles_per_unit;
        const int bh = quot(u, p.qI), i = u - bh * p.I;
        const int b = quot(bh, p.qHkv), h = bh - b * p.Hkv;
        const int r = unit_row(b * p.I + i, p.UPBs, G) + r16;
        const int j = jt * 16 + 4 * kg;
        uint32_t w[2];
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
            const uint32_t lo = (j + e < p.m) ? f32_to_bf16_bits(acc[e] * p.scale) : 0u;
            const uint32_t hi = (j + e + 1 < p.m) ? f32_to_bf16_bits(acc[e + 1] * p.scale) : 0u;
            w[e >> 1] = lo | (hi << 16);
        }
        uint16_t *srow = p.S + (static_cast<size_t>(h) * p.R_pad + r) * p.m_pad + j;
        *reinterpret_cast<u32x2 *>(srow) = u32x2_mk(w[0], w[1]);
        // the consumer reads whole 32-wide k-steps: keep the padding [m16, m_pad) at zero
        if (jt == p.tiles_per_unit - 1 && p.m_pad > p.m16) *reinterpret_cast<u32x2 *>(srow + 16) = u32x2_mk(0u, 0u);
    }
    TS(0, 4);
}

// ------------------------------------------------------------------------------------------
// Pieces of Alg. 1 step 2 shared by fb_probs and fab_fused (which runs them behind its own first
// phase): L[r][pos] = sum_j S[r][j] theta[j][pos] for one tile of 16 NW rows x 64 positions, then
// P = exp(L - tile max).  MFMA tile: A = theta^T (16 positions x 32 j) from LDS, B = S^T (32 j x 16
// rows) from memory, D[pos][row]: a lane ends up with 4 consecutive positions of one row.
// ------------------------------------------------------------------------------------------
// The theta chunk [m x 64 positions] goes to LDS transposed (ThT[pos][j], rows LDT apart).  A thread
// owns a pair of consecutive rows j, j+1 and 8 positions; the pair is packed so the transposed store
// is one 32-bit word per position.
template <int KS4, int NW> struct ThetaChunk {
    static constexpr int RPP = 16 * NW;              // rows of theta per pass of the workgroup
    static constexpr int FB = 128 * KS4 / RPP;       // passes of RPP rows: RPP FB >= m_pad, all in one batch
    u32x4 tv[FB][2];
    int seg, j0;                                      // 16-byte segment of the chunk row; first row of the pair

    __device__ __forceinline__ void request(const Plan &p, const uint16_t *__restrict__ theta, int h, int pc, int wave, int lane)
    {
        seg = (lane >> 4) + 4 * (wave & 1);
        j0 = 2 * ((lane & 15) + 16 * (wave >> 1));
        const uint16_t *th = theta + static_cast<size_t>(h) * p.m * p.n + pc * kPC + 8 * seg;
#pragma unroll
        for (int k = 0; k < FB; ++k)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                // no run-time test around the loads (they would be waited for on the spot): rows beyond m are
                // clamped to the last one here and replaced by zeros where they are stored
                const int j = j0 + RPP * k + e;
                tv[k][e] = *reinterpret_cast<const u32x4 *>(th + static_cast<size_t>(min(j, p.m - 1)) * p.n);
            }
    }

    __device__ __forceinline__ void store(const Plan &p, uint16_t *ThT, int LDT) const
    {
#pragma unroll
        for (int k = 0; k < FB; ++k) {
            const int j = j0 + RPP * k;
            if (j < p.m16) {
                const uint32_t ka = j < p.m ? 0xffffffffu : 0u, kc = j + 1 < p.m ? 0xffffffffu : 0u;
                const uint32_t a[4] = {tv[k][0].x & ka, tv[k][0].y & ka, tv[k][0].z & ka, tv[k][0].w & ka};
                const uint32_t c[4] = {tv[k][1].x & kc, tv[k][1].y & kc, tv[k][1].z & kc, tv[k][1].w & kc};
                uint32_t *dst = reinterpret_cast<uint32_t *>(ThT + (8 * seg) * LDT + j);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    dst[(2 * e) * (LDT / 2)] = (a[e] & 0xffffu) | (c[e] << 16);
                    dst[(2 * e + 1) * (LDT / 2)] = (a[e] >> 16) | (c[e] & 0xffff0000u);
                }
            }
        }
        // zero the k padding of the transposed chunk: columns [m16, m_pad)
        const int padc = p.m_pad - p.m16;
        for (int idx = threadIdx.x; idx < kPC * padc; idx += 64 * NW) {
            const int pp = idx / padc, j = p.m16 + idx - pp * padc;
            ThT[pp * LDT + j] = 0;
        }
    }
};

// The scores of row r as MFMA B fragments, KS = m_pad / 32 k-steps of 32 compressed positions handled
// as KS4 groups of four without any test inside the loops.  A step of the last group that lies beyond
// KS re-reads the last step and is masked where it is used: loads under a run-time test, even a
// uniform one, made the compiler wait for each of them in turn and shuttle the fragments through
// accumulator registers when KS4 = 2; an assignment of zeros under a test lets the compiler move the
// load under the test again.  Every lane loads, also in a wave whose rows lie beyond R: they exist in
// the workspace up to R_pad, and nothing of such a wave is stored.
template <int KS4> __device__ __forceinline__ void request_scores(u32x4 (&sfr)[4 * KS4], const Plan &p, int h, int r, int kg)
{
    constexpr int SB = 4 * KS4;
    const int KS = p.m_pad / 32;
    const uint16_t *srow = p.S + (static_cast<size_t>(h) * p.R_pad + r) * p.m_pad + 8 * kg;
#pragma unroll
    for (int k = 0; k < SB; ++k) {
        sfr[k] = *reinterpret_cast<const u32x4 *>(srow + 32 * (k < SB - 4 ? k : min(k, KS - 1)));
        // the first eight are requested here: left alone, the instruction scheduler spreads the loads over
        // the matrix work below, a few at a time, and every one becomes a round trip of its own
        if (k == (SB < 8 ? SB : 8) - 1) __builtin_amdgcn_sched_barrier(0);
    }
}

// L for the wave's 16 rows x 64 positions, the tile-local softmax numerators in bf16 and the tile's
// (max, sum) per row; KID names the kernel in the developer timeline.
template <int KS4, int KID>
__device__ __forceinline__ void probs_tile(const Plan &p, const uint16_t *ThT, int LDT, const u32x4 (&sfr)[4 * KS4], int h, int r,
                                           int pc, int r16, int kg)
{
    constexpr int SB = 4 * KS4, PC = kPC;
    const int KS = p.m_pad / 32;
    f32x4 acc[PC / 16];
#pragma unroll
    for (int mt = 0; mt < PC / 16; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < SB; ++k) {
        const int ks = min(k, KS - 1);
        // scores beyond the compressed length are zeros written with the scores
        const uint32_t keep = (k < SB - 4 || k < KS) ? 0xffffffffu : 0u;
        const bf16x8 bfrag = as_bf16x8(u32x4_mk(sfr[k].x & keep, sfr[k].y & keep, sfr[k].z & keep, sfr[k].w & keep));
#pragma unroll
        for (int mt = 0; mt < PC / 16; ++mt) {
            const bf16x8 afrag = *reinterpret_cast<const bf16x8 *>(ThT + (16 * mt + r16) * LDT + 32 * ks + 8 * kg);
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, bfrag, acc[mt], 0, 0, 0);
        }
    }

    TS(KID, 3);
    // ---- tile-local softmax numerators of row r over the 64 positions ------------------------------
    float mx = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < PC / 16; ++mt)
#pragma unroll
        for (int e = 0; e < 4; ++e) mx = fmaxf(mx, acc[mt][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    float sum = 0.f;
    const bool valid = row_valid(p, r);
    uint16_t *prow = p.P + (static_cast<size_t>(h) * p.R_pad + r) * p.n + pc * PC + 4 * kg;
#pragma unroll
    for (int mt = 0; mt < PC / 16; ++mt) {
        const uint32_t a0 = f32_to_bf16_bits(__expf(acc[mt][0] - mx)), a1 = f32_to_bf16_bits(__expf(acc[mt][1] - mx));
        const uint32_t a2 = f32_to_bf16_bits(__expf(acc[mt][2] - mx)), a3 = f32_to_bf16_bits(__expf(acc[mt][3] - mx));
        sum += __uint_as_float(a0 << 16) + __uint_as_float(a1 << 16) + __uint_as_float(a2 << 16) + __uint_as_float(a3 << 16);
        if (valid) *reinterpret_cast<u32x2 *>(prow + 16 * mt) = u32x2_mk(a0 | (a1 << 16), a2 | (a3 << 16));
    }
    sum += __shfl_xor(sum, 16, 64);
    sum += __shfl_xor(sum, 32, 64);
    if (kg == 0 && valid) p.stats[(static_cast<size_t>(h) * p.R_pad + r) * p.NC + pc] = f32x2_mk(mx, sum);
    TS(KID, 4);
}

// ------------------------------------------------------------------------------------------
// fb_probs: Alg. 1 step 2 and the numerator of the softmax for one tile of 16 NW rows x 64
// positions (NW waves, one 16-row MFMA tile each), from the pieces above.
// ------------------------------------------------------------------------------------------
// The leading arguments repeat what stands in front of the first loads (14 dwords: the hardware
// hands them to every wave in registers at its start); the rest of the plan is fetched behind them.
template <int KS4, int NW>
__global__ __launch_bounds__(64 * NW) void fb_probs(const uint16_t *__restrict__ theta, uint16_t *a_S, unsigned a_qNC,
                                                    int a_NC, unsigned a_qHkv, int a_Hkv, int a_NRB, int a_R, int a_R_pad,
                                                    int a_m_pad, int a_m, int a_n, Plan p)
{
    p.S = a_S; p.qNC = a_qNC; p.NC = a_NC; p.qHkv = a_qHkv; p.Hkv = a_Hkv; p.NRB = a_NRB; p.R = a_R;
    p.R_pad = a_R_pad; p.m_pad = a_m_pad; p.m = a_m; p.n = a_n;
    extern __shared__ __align__(16) uint16_t lds[];
    constexpr int PC = kPC;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, kg = lane >> 4;

    // Workgroup ids are dealt round-robin over the 8 XCDs (private L2s).  The pair (row block rb,
    // head h) picks the XCD (key = h + H_kv rb, class key mod 8): its rows of S reach one L2 only,
    // and a chunk of theta[h] at most 8 / H_kv of them.
    const int w8 = blockIdx.x >> 3;
    const int w8q = quot(w8, p.qNC);
    const int pc = w8 - w8q * p.NC, key = w8q * 8 + (blockIdx.x & 7);
    if (key >= p.NRB * p.Hkv) return;
    const int rb = quot(key, p.qHkv), h = key - rb * p.Hkv;

    TS(1, 0);
    const int LDT = p.m_pad + 8;
    uint16_t *ThT = lds;                 // [PC][LDT]   theta chunk, transposed: ThT[pos][j]

    // scores of this wave's 16 rows: first batch of fragments in flight during the LDS fill
    const int r0 = rb * (16 * NW) + wave * 16;
    const bool wave_live = r0 < p.R;
    const int r = r0 + r16;
    u32x4 sfr[4 * KS4];
    request_scores<KS4>(sfr, p, h, r, kg);

    TS(1, 1);
    ThetaChunk<KS4, NW> th;
    th.request(p, theta, h, pc, wave, lane);
    fetch_now(p.m16, p.P, p.stats);
    th.store(p, ThT, LDT);
    __syncthreads();
    TS(1, 2);
    if (!wave_live) return;
    probs_tile<KS4, 1>(p, ThT, LDT, sfr, h, r, pc, r16, kg);
}

// ------------------------------------------------------------------------------------------
// fab_fused: fa_scores and fb_probs in one launch, for calls small enough that all its workgroups are
// resident at once.  The NC chunk workgroups of a (head, 64-row block) pair first compute the pair's
// rows of S between them (up to TQ tiles of 16 key rows per wave, streamed from HBM while the theta
// chunk arrives from the L2), then hand them to each other through the L2: a workgroup waits until
// its stores are acknowledged, adds one to the pair's counter and polls it (with an atomic add of
// zero, which is carried out in the L2 -- a plain load may be answered by the CU's L1) until all NC
// have arrived, invalidates its L1 and goes on as fb_probs.
//  * Workgroup ids of one residue class mod 8 run on one XCD, and a pair's workgroups share a class
//    (see fb_probs), so counter and data meet in one L2 and neither a write-back nor an invalidation
//    of it is needed.  This is a matter of speed only: atomics without device scope stay in the
//    issuing XCD's L2, so a counter can reach NC only through workgroups that share that L2 -- and
//    then their data is there too.
//  * A workgroup that does not see NC arrivals within p.wait_ticks (siblings not resident, or on
//    another XCD) computes all of the pair's rows of S itself and reads those: slower, same result
//    (a debug counter records it).
//  * The counters live at the start of the caller's workspace as (epoch, count) words (see ctr_claim):
//    nothing has to be initialised, nothing is shared between calls that use different workspaces, and
//    the finalize kernel of the same call puts them back to zero.
// ------------------------------------------------------------------------------------------
template <int KS4, int G>
__global__ __launch_bounds__(256) void fab_fused(const uint16_t *__restrict__ Kc, u64 *a_flags, unsigned a_qNC, int a_NC, unsigned a_qHkv,
                                                 int a_Hkv, int a_nkeys, int a_TPU, unsigned a_qTPU, int a_UPBs, int a_I,
                                                 unsigned a_qI, int a_m, int a_units, Plan p,
                                                 const uint16_t *__restrict__ theta, const uint16_t *__restrict__ q)
{
    constexpr int NW = 4, TQ = 4;
    p.qNC = a_qNC; p.NC = a_NC; p.qHkv = a_qHkv; p.Hkv = a_Hkv; p.tiles_per_unit = a_TPU; p.qTPU = a_qTPU;
    p.UPBs = a_UPBs; p.I = a_I; p.qI = a_qI; p.m = a_m;
    extern __shared__ __align__(16) uint16_t lds[];
    constexpr int PC = kPC;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, kg = lane >> 4;

    // Workgroup ids are dealt round-robin over the 8 XCDs (private L2s).  The pair (row block rb,
    // head h) picks the XCD (key = h + H_kv rb, class key mod 8): its rows of S reach one L2 only,
    // and a chunk of theta[h] at most 8 / H_kv of them.
    const int w8 = blockIdx.x >> 3;
    const int w8q = quot(w8, p.qNC);
    const int pc = w8 - w8q * p.NC, key = w8q * 8 + (blockIdx.x & 7);
    if (key >= a_nkeys) return;
    const int rb = quot(key, p.qHkv), h = key - rb * p.Hkv;
    u64 *flag = a_flags + static_cast<size_t>(key) * kCtrStride;

    // ---- phase 1: this workgroup's share of S = sigma q Kc^T for the pair's image blocks ---------------
    // tiles of 16 key rows are numbered (image block of the row block, tile of the block); wave w takes
    // tiles pc TW + w + 4 t; a tile beyond the share repeats the last one and is not stored
    // (T counts the tiles of the image blocks the row block really has)
    const int T = a_TPU * min(1 << a_UPBs, a_units - (rb << a_UPBs)), TW = quot(T + a_NC - 1, a_qNC);
    // one tile of S: lane (head r16, key rows 4 kg ..) of image block ub, tile jt
    auto store_tile = [&](const f32x4 &sacc, int ub, int jt) {
        if (r16 >= G) return;                // columns beyond the group are copies of head G-1
        const int rr = unit_row(ub, a_UPBs, G) + r16, j = jt * 16 + 4 * kg;
        uint32_t wv[2];
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
            const uint32_t lo2 = (j + e < p.m) ? f32_to_bf16_bits(sacc[e] * p.scale) : 0u;
            const uint32_t hi2 = (j + e + 1 < p.m) ? f32_to_bf16_bits(sacc[e + 1] * p.scale) : 0u;
            wv[e >> 1] = lo2 | (hi2 << 16);
        }
        uint16_t *sr = p.S + (static_cast<size_t>(h) * p.R_pad + rr) * p.m_pad + j;
        *reinterpret_cast<u32x2 *>(sr) = u32x2_mk(wv[0], wv[1]);
        // the consumer reads whole 32-wide k-steps: keep the padding [m16, m_pad) at zero
        if (jt == a_TPU - 1 && p.m_pad > p.m16) *reinterpret_cast<u32x2 *>(sr + 16) = u32x2_mk(0u, 0u);
    };
    u32x4 kf[TQ][4];
    int t_ub[TQ], t_jt[TQ];
    bool t_live[TQ];
#pragma unroll
    for (int tq = 0; tq < TQ; ++tq) {
        const int tw = wave + 4 * tq, tl = min(pc * TW + min(tw, TW - 1), T - 1);
        const int k = quot(tl, a_qTPU), jt = tl - k * a_TPU;
        const int ub = min((rb << a_UPBs) + k, a_units - 1);
        t_live[tq] = tw < TW && pc * TW + tw < T && (rb << a_UPBs) + k < a_units;
        t_ub[tq] = ub; t_jt[tq] = jt;
        const int b = quot(ub, a_qI), i = ub - b * a_I;
        const int u = (b * a_Hkv + h) * a_I + i;
        const int row = min(jt * 16 + r16, a_m - 1);
        const u32x4 *kp = reinterpret_cast<const u32x4 *>(Kc + (static_cast<size_t>(u) * a_m + row) * D) + kg;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) kf[tq][ks] = kp[4 * ks];
    }
    fetch_now(theta, q, p.Hq, p.n, p.m_pad);
    u32x4 qf[TQ][4];
#pragma unroll
    for (int tq = 0; tq < TQ; ++tq) {
        const int b = quot(t_ub[tq], a_qI);
        const u32x4 *qp = reinterpret_cast<const u32x4 *>(q + (static_cast<size_t>(b) * p.Hq + h * G + min(r16, G - 1)) * D) + kg;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qf[tq][ks] = qp[4 * ks];
    }

    TS(1, 0);
    const int LDT = p.m_pad + 8;
    uint16_t *ThT = lds;                 // [PC][LDT]   theta chunk, transposed: ThT[pos][j]

    TS(1, 1);
    // the theta chunk is requested before the score tiles are multiplied and stored to LDS after them
    ThetaChunk<KS4, NW> th;
    th.request(p, theta, h, pc, wave, lane);
    fetch_now(p.m16, p.P, p.stats, p.S, p.scale, p.R_pad, p.R, p.RV, p.epoch, p.wait_ticks, p.fallbacks);
    // thread 0 raises the pair's counter word to this call's epoch (behind the loads above, so that it does
    // not stand in front of them; measured: 0.3 us per call better here than next to the wait below)
    if (threadIdx.x == 0) ctr_claim(flag, p.epoch);
    // S tiles of this wave
#pragma unroll
    for (int tq = 0; tq < TQ; ++tq) {
        f32x4 sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kf[tq][ks]), as_bf16x8(qf[tq][ks]), sacc, 0, 0, 0);
        if (t_live[tq]) store_tile(sacc, t_ub[tq], t_jt[tq]);
    }
    th.store(p, ThT, LDT);
    // every wave's stores of S (and thread 0's claim of the counter word) have been acknowledged by the L2
    // before the counter moves
    __shared__ int sAlone;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(flag, static_cast<u64>(1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        const u64 want = ctr_word(p.epoch, static_cast<unsigned>(a_NC));
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
    __syncthreads();
    if (sAlone) {
        // nobody to rely on: all T tiles of the pair, 16 per round (a wave takes tiles base + w + 4 t)
        for (int base = 0; base < T; base += 16) {
            for (int tq = 0; tq < 4; ++tq) {
                const int tl = base + wave + 4 * tq;
                if (tl >= T) continue;
                const int k = quot(tl, a_qTPU), jt = tl - k * a_TPU;
                const int ub = (rb << a_UPBs) + k;
                if (ub >= a_units) continue;
                const int b = quot(ub, a_qI), i = ub - b * a_I;
                const int u = (b * a_Hkv + h) * a_I + i;
                const u32x4 *kp = reinterpret_cast<const u32x4 *>(Kc + (static_cast<size_t>(u) * a_m + min(jt * 16 + r16, a_m - 1)) * D) + kg;
                const u32x4 *qp = reinterpret_cast<const u32x4 *>(q + (static_cast<size_t>(b) * p.Hq + h * G + min(r16, G - 1)) * D) + kg;
                f32x4 sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kp[4 * ks]), as_bf16x8(qp[4 * ks]), sacc, 0, 0, 0);
                store_tile(sacc, ub, jt);
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }
    asm volatile("buffer_inv sc0" ::: "memory");
    TS(1, 2);
    const int r0 = rb * (16 * NW) + wave * 16;
    const int r = r0 + r16;
    u32x4 sfr[4 * KS4];
    request_scores<KS4>(sfr, p, h, r, kg);
    if (r0 >= p.R) return;
    probs_tile<KS4, 1>(p, ThT, LDT, sfr, h, r, pc, r16, kg);
}

// ------------------------------------------------------------------------------------------
// fc_fused: Alg. 1 steps 3 and 4 on 64 rows of U / Vc for a group of query rows.
// G query heads per KV head; a workgroup handles NT MFMA tiles of 16 query rows, each tile
// holding UP whole image blocks (G * UP <= 16); NC = n / 64 softmax tiles per image block
// (compile time, so that every loop below is free of bounds checks).
// 8 waves: wave w = (kh, jt) owns rows j = lo + 16 jt .. + 15 of U and the tiles
// [kh ? KH0 : 0, kh ? NC : KH0) of the positions for step 3 (the two halves are added through
// LDS), and channels 16 w .. 16 w + 15 for step 4.
// Part record in Ypart: [G][D] floats of un-normalised output, [G] maxima, [G] sums.
// ------------------------------------------------------------------------------------------
template <int NC> struct KSplit;          // tiles of k-half 0, tiles staged per step
template <> struct KSplit<16> { static constexpr int KH0 = 8, UCH = 4; };
template <> struct KSplit<9> { static constexpr int KH0 = 6, UCH = 3; };
template <> struct KSplit<4> { static constexpr int KH0 = 2, UCH = 2; };

// (leading arguments: what stands in front of the first loads, preloaded into registers, see fb_probs)
template <int G, int UP, int NT, int NC, bool RAG>
__global__ __launch_bounds__(512) void fc_fused(const uint16_t *__restrict__ U, uint16_t *a_P, f32x2 *a_stats,
                                                unsigned a_qJS, int a_JS, unsigned a_qHkv, int a_Hkv, int a_B, int a_I,
                                                int a_m, int a_UPBs_pk, Plan p,
                                                const uint16_t *__restrict__ Vc,
                                                const uint16_t *__restrict__ q,
                                                uint16_t *__restrict__ Kt, uint16_t *__restrict__ Vt,
                                                const uint16_t *__restrict__ k_new,
                                                const uint16_t *__restrict__ v_new)
{
    static_assert(G * UP <= 16, "the rows of a tile must fit one MFMA tile");
    // (bit 8 of this preloaded argument: U comes in the packed form of kvc_pack_u)
    const int a_UPBs = a_UPBs_pk & 255;
    const bool upk = (a_UPBs_pk >> 8) != 0;
    p.P = a_P; p.stats = a_stats; p.qJS = a_qJS; p.JS = a_JS; p.qHkv = a_qHkv; p.Hkv = a_Hkv; p.B = a_B; p.I = a_I;
    p.m = a_m;
    p.R_pad = (unit_row(a_B * a_I - 1, a_UPBs, G) + G + kRB - 1) & ~(kRB - 1);
    // as the host computes them
    p.NG = (a_B * a_I + NT * UP - 1) / (NT * UP);
    p.nvis_c = ((p.NG * a_Hkv + 7) & ~7) * a_JS;
    constexpr int n = NC * kPC, LDP = n + 8;
    constexpr int NR = 16 * NT;
    constexpr int NU = NT * UP;                          // image blocks per workgroup
    constexpr int KH0 = KSplit<NC>::KH0, UCH = KSplit<NC>::UCH;
    constexpr int NSTEP = KH0 / UCH;                     // steps of the longer k-half
    extern __shared__ __align__(16) uint16_t dyn[];      // P [NR][LDP], then the partial sums of k-half 1
    __shared__ __align__(16) uint16_t sWb[NR][kWLD];     // W tile, bf16
    __shared__ float sAl[NR][NC + 1];                    // alpha[row][tile]
    __shared__ float sMx[NR], sSm[NR];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, kg = lane >> 4;
    const int jt = wave & 3, kh = wave >> 2;

    // Workgroup ids are dealt round-robin over the 8 XCDs (private L2s).  The pair (row group ug,
    // head h) picks the XCD: key = h + H_kv ug, class key mod 8; the JS slices of one pair share a
    // class, so its rows of P are fetched into one L2 only, and the rows of U[h] into at most
    // 8 / H_kv of them (one when H_kv >= 8).
    // The text chunks ride along as the last workgroups (four waves each): they land on the CUs the
    // others leave idle first, and end before the longest of the others does.
    if (static_cast<int>(blockIdx.x) >= p.nvis_c) {
        if (threadIdx.x < 256) text_part<G, RAG>(p, q, Kt, Vt, k_new, v_new, dyn, blockIdx.x - p.nvis_c, threadIdx.x, true);
        return;
    }
    TS(2, 0);
    const int w8 = blockIdx.x >> 3;
    const int w8q = quot(w8, p.qJS);
    const int s = w8 - w8q * p.JS, key = w8q * 8 + (blockIdx.x & 7);
    if (key >= p.NG * p.Hkv) return;
    const int ug = quot(key, p.qHkv), h = key - ug * p.Hkv;
    const int ub0 = ug * NU;
    const int units_total = p.B * p.I;
    const int nunits = min(NU, units_total - ub0);
    // the workgroup's image blocks are consecutive rows of one 64-row block: 64 / G rounded down to a
    // multiple of the 2 UP blocks of two tiles, always a power of two for the compiled group sizes
    const int row0 = unit_row(ub0, a_UPBs, G);
    const int lo = s * kJC, hi = min(p.m, lo + kJC);
    uint16_t *sP = dyn;

    // ---- everything this workgroup reads is requested up front, without bounds checks: -----------------
    // out-of-range rows are clamped to valid ones and their results are never stored
    // P rows -> LDS: 16 threads per row, 32 rows per pass
    constexpr int PCH = n / 8;                           // 16-byte pieces per row
    constexpr int KP = (PCH + 15) / 16;
    constexpr int NPASS = (NR + 31) / 32;                // passes of 32 rows
    u32x4 pfr[NPASS][KP];
    const int prow_i = threadIdx.x >> 4, psub = threadIdx.x & 15;
#pragma unroll
    for (int ps = 0; ps < NPASS; ++ps) {
        const int pr = min(prow_i + 32 * ps, NR - 1);
        const int r = row0 + min((pr >> 4) * (UP * G) + min(pr & 15, UP * G - 1), nunits * G - 1);
        const u32x4 *prow = reinterpret_cast<const u32x4 *>(p.P + (static_cast<size_t>(h) * p.R_pad + r) * n);
#pragma unroll
        for (int k = 0; k < KP; ++k) pfr[ps][k] = prow[min(16 * k + psub, PCH - 1)];
    }
    // image blocks a sequence of a ragged batch does not have (block i >= its count): bit un of `present`
    // is clear; their rows of P and statistics are replaced by "no mass" below and their outputs dropped,
    // whatever the capsule slot and the earlier kernels left there
    static_assert(NU <= 64, "one bit per image block of the workgroup");
    // (a uniform call has them all: the mask is a constant and every test on it folds away)
    unsigned long long present = ~0ull;
    if constexpr (RAG) {
        // lane un of every wave looks its block up; the wave's ballot is the mask
        const int ub = ub0 + min(lane, nunits - 1);
        const int b = quot(ub, p.qI), i = ub - b * p.I;
        present = __ballot(i < p.n_img[b]);
    }
    // image block (within the workgroup) of row pr of the workgroup's NR rows
    auto unit_of = [&](int pr) { return (pr >> 4) * UP + min(pr & 15, UP * G - 1) / G; };
    // tile statistics: lane (kg = MFMA tile, r16 = row) of wave 0 reads one f32x2 per softmax tile
    f32x2 st[NC];
#pragma unroll
    for (int k = 0; k < NC; ++k) st[k] = f32x2_mk(0.f, 0.f);
    if (wave == 0) {
        const int r = row0 + min(min(kg, NT - 1) * (UP * G) + min(r16, UP * G - 1), nunits * G - 1);
        const f32x2 *sp = p.stats + (static_cast<size_t>(h) * p.R_pad + r) * NC;
#pragma unroll
        for (int k = 0; k < NC; ++k) st[k] = sp[k];
    }
    // U rows lo + 16 jt ... of this wave's tiles, fully coalesced: 8 lanes read the 128 bytes of one
    // row of one tile, 8 rows per instruction; all steps stay in flight
    const int c_begin = kh ? KH0 : 0;
    const int nstep = kh ? (NC - KH0) / UCH : NSTEP;
    // Only the first step's rows are requested here; the next step and the compressed values follow
    // once the matrix work has started, so that the loads of one wave overlap the MFMAs of the other
    // wave on its SIMD instead of holding up the instruction stream in front of them.
    u32x4 ul[NSTEP][2 * UCH];
    // rows of U as MFMA operands straight from memory: lane (r16, kg) reads 16 bytes of row r16
    // (plain form: 16 bytes of row r16 at position 8 kg of the tile; packed form: blocks of 8 positions, each [m][8],
    // in which the 16-byte pieces of the 16 rows are adjacent and a quarter-wave reads two whole lines)
    const int urow = min(lo + 16 * jt + r16, p.m - 1);
    const uint16_t *ud = upk ? U + static_cast<size_t>(h) * p.m * n + (static_cast<size_t>(c_begin * (kPC / 8) + kg) * p.m + urow) * 8
                             : U + (static_cast<size_t>(h) * p.m + urow) * n + c_begin * kPC + 8 * kg;
    const int u_tile = upk ? kPC * p.m : kPC, u_half = upk ? 32 * p.m : 32;     // elements from tile to tile, to the second k-step
    auto load_u = [&](int step) {
        // a step the shorter k-half does not have re-reads its last tile; the result is not used
        const int cs0 = min(step, nstep - 1) * UCH;
#pragma unroll
        for (int ci = 0; ci < UCH; ++ci) {
            ul[step][2 * ci] = *reinterpret_cast<const u32x4 *>(ud + static_cast<size_t>(cs0 + ci) * u_tile);
            ul[step][2 * ci + 1] = *reinterpret_cast<const u32x4 *>(ud + static_cast<size_t>(cs0 + ci) * u_tile + u_half);
        }
    };
    load_u(0);
    fetch_now(Vc, p.Ypart, p.nparts, p.rec, p.merge, p.qI, p.n_img);
    // compressed values: wave w owns channels 16 w ...; the operand (8 rows j of one channel) is 16
    // contiguous bytes in the blocked layout.  Image blocks are handled in batches of UBATCH.
    constexpr int UBATCH = NU < 4 ? NU : 4;
    const int jb0 = lo >> 3;
    const int nfull = p.m >> 3;                          // complete 8-row blocks of a record
    const int wtail = p.m & 7;
    const bool has_tail = wtail != 0 && hi == p.m;       // the shorter last block lives in the last slice
    const int cch = 16 * wave + r16;                     // this lane's channel
    // Every lane issues the same two 16-byte loads per image block whatever the slice holds (loads under a
    // run-time test would be waited for on the spot).  Where a lane's 8-row block is the shorter last one,
    // [D][wtail], its wtail values are 2 wtail consecutive bytes of that block: the lane reads the 16-byte
    // window around them (dword aligned, kept inside the block) and shift_tail() moves them into place
    // once the data is there.  Blocks beyond the record are clamped to a valid one, a record shorter than
    // one block reads its first 16 bytes; whatever lies in rows j >= m meets a zero weight in W.
    const int tail_off = cch * 2 * wtail;
    const int tail_a0 = max(min(tail_off & ~3, D * 2 * wtail - 16), 0);
    const int tail_sh = tail_off - tail_a0;              // 0 .. 14, even; tail_sh + 2 wtail <= 16
    const int lb = nfull - jb0;                          // the short block's place in this slice: k-step lb / 4, lanes kg == lb % 4
    uint32_t voffb[2];                                   // byte offsets into a record
    int tail_ds[2];                                      // whole dwords to shift by (0 for every other lane)
    uint32_t tail_bs[2];                                 // then 0 or 16 bits
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int jbq = jb0 + 4 * ks + kg;
        const bool mine = has_tail && jbq == nfull;
        const int jb = min(jbq, max(nfull - 1, 0));
        voffb[ks] = mine ? static_cast<uint32_t>(nfull * 8 * D * 2 + tail_a0)
                         : (nfull > 0 ? static_cast<uint32_t>(jb * 8 * D * 2 + cch * 16) : 0u);
        tail_ds[ks] = mine ? tail_sh >> 2 : 0;
        tail_bs[ks] = mine ? (tail_sh & 2) * 8u : 0u;
    }
    auto load_values = [&](int un0, u32x4 (&dst)[UBATCH][2]) {
#pragma unroll
        for (int a = 0; a < UBATCH; ++a) {
            const int ub = ub0 + min(un0 + a, nunits - 1);
            const int b = quot(ub, p.qI), i = ub - b * p.I;
            const char *vbase = reinterpret_cast<const char *>(Vc + (static_cast<size_t>(b * p.Hkv + h) * p.I + i) * p.m * D);
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) dst[a][ks] = *reinterpret_cast<const u32x4_a4 *>(vbase + voffb[ks]);
        }
    };
    // 128-bit right shift of the windows of the short block (registers only; other lanes shift by nothing)
    auto shift_tail = [&](u32x4 (&v)[UBATCH][2]) {
        if (!has_tail) return;
#pragma unroll
        for (int a = 0; a < UBATCH; ++a)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                if (ks != (lb >> 2)) continue;
                const u32x4 wv = v[a][ks];
                const bool d1 = tail_ds[ks] & 1, d2 = tail_ds[ks] & 2;
                const uint32_t y0 = d1 ? wv.y : wv.x, y1 = d1 ? wv.z : wv.y, y2 = d1 ? wv.w : wv.z, y3 = d1 ? 0u : wv.w;
                const uint32_t x0 = d2 ? y2 : y0, x1 = d2 ? y3 : y1, x2 = d2 ? 0u : y2, x3 = d2 ? 0u : y3;
                v[a][ks] = u32x4_mk(__builtin_amdgcn_alignbit(x1, x0, tail_bs[ks]), __builtin_amdgcn_alignbit(x2, x1, tail_bs[ks]),
                                    __builtin_amdgcn_alignbit(x3, x2, tail_bs[ks]), x3 >> tail_bs[ks]);
            }
    };
    // one batch of image blocks is in flight ahead of the one being multiplied (two ahead measured no
    // better: their registers cost a resident workgroup per CU)
    constexpr int NBATCH = NU / UBATCH;
    constexpr int DEPTH = 1;
    static_assert(NU % UBATCH == 0, "whole batches");
    u32x4 vfr[DEPTH + 1][UBATCH][2];

    TS(2, 1);
    // ---- block statistics: alpha[row][tile] = exp(tile max - block max) ----------------------------------
    if (wave == 0 && kg < NT) {
        if (!((present >> unit_of(16 * kg + r16)) & 1ull)) {
#pragma unroll
            for (int k = 0; k < NC; ++k) st[k] = f32x2_mk(-1e30f, 0.f);
        }
        float mx = st[0].x;
#pragma unroll
        for (int k = 1; k < NC; ++k) mx = fmaxf(mx, st[k].x);
        float sm = 0.f;
#pragma unroll
        for (int k = 0; k < NC; ++k) {
            const float a = __expf(st[k].x - mx);
            sm += st[k].y * a;
            sAl[16 * kg + r16][k] = a;
        }
        sMx[16 * kg + r16] = mx;
        sSm[16 * kg + r16] = sm;
    }
#pragma unroll
    for (int ps = 0; ps < NPASS; ++ps)
        if (prow_i + 32 * ps < NR) {
            u32x4 *dst = reinterpret_cast<u32x4 *>(sP + (prow_i + 32 * ps) * LDP);
            const unsigned keep = ((present >> unit_of(prow_i + 32 * ps)) & 1ull) ? 0xffffffffu : 0u;
#pragma unroll
            for (int k = 0; k < KP; ++k)      // clamped duplicates carry equal data
                dst[min(16 * k + psub, PCH - 1)] = u32x4_mk(pfr[ps][k].x & keep, pfr[ps][k].y & keep, pfr[ps][k].z & keep, pfr[ps][k].w & keep);
        }
    __syncthreads();
    TS(2, 2);

    // ---- step 3: W^T[j][row] = sum_tiles alpha[row][tile] sum_pos U[j][pos] P[row][pos] ------------------
    f32x4 w[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) w[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    {
        const uint16_t *pb = sP + r16 * LDP + 8 * kg + c_begin * kPC;
        const float *al = &sAl[r16][c_begin];
#pragma unroll
        for (int step = 0; step < NSTEP; ++step) {
            if (step + 1 < NSTEP) load_u(step + 1);
            if (step == NSTEP - 1) load_values(0, vfr[0]);
            if (step < nstep) {
#pragma unroll
                for (int ci = 0; ci < UCH; ++ci) {      // one softmax tile = 64 positions = two k-steps
                    const int c = step * UCH + ci;
                    const bf16x8 a0 = as_bf16x8(ul[step][2 * ci]), a1 = as_bf16x8(ul[step][2 * ci + 1]);
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        f32x4 wt = {0.f, 0.f, 0.f, 0.f};
                        wt = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            a0, *reinterpret_cast<const bf16x8 *>(pb + 16 * t * LDP + kPC * c), wt, 0, 0, 0);
                        wt = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            a1, *reinterpret_cast<const bf16x8 *>(pb + 16 * t * LDP + kPC * c + 32), wt, 0, 0, 0);
                        const float a = al[16 * t * (NC + 1) + c];
                        w[t][0] += a * wt[0]; w[t][1] += a * wt[1]; w[t][2] += a * wt[2]; w[t][3] += a * wt[3];
                    }
                }
            }
        }
    }
    // the two k-halves meet in LDS: half 1 parks its partial sums behind the rows of P
    f32x4 *park = reinterpret_cast<f32x4 *>(dyn + NR * LDP) + jt * (64 * NT) + lane;
    if (kh == 1) {
#pragma unroll
        for (int t = 0; t < NT; ++t) park[64 * t] = f32x4_mk(w[t][0], w[t][1], w[t][2], w[t][3]);
    }
    __syncthreads();
    if (kh == 0) {
        const int jl = 16 * jt + 4 * kg;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const f32x4 o = park[64 * t];
            const float w0 = w[t][0] + o.x, w1 = w[t][1] + o.y, w2 = w[t][2] + o.z, w3 = w[t][3] + o.w;
            const uint32_t b0 = (lo + jl + 0 < hi) ? f32_to_bf16_bits(w0) : 0u, b1 = (lo + jl + 1 < hi) ? f32_to_bf16_bits(w1) : 0u;
            const uint32_t b2 = (lo + jl + 2 < hi) ? f32_to_bf16_bits(w2) : 0u, b3 = (lo + jl + 3 < hi) ? f32_to_bf16_bits(w3) : 0u;
            *reinterpret_cast<u32x2 *>(&sWb[16 * t + r16][jl]) = u32x2_mk(b0 | (b1 << 16), b2 | (b3 << 16));
        }
    }
    __syncthreads();
    TS(2, 3);

    // ---- step 4: out_part^T[c][row] = sum_j Vc^T[c][j] W[row][j], per image block -------------------------
    bf16x8 wb[NT][2];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        wb[t][0] = *reinterpret_cast<const bf16x8 *>(&sWb[16 * t + r16][8 * kg]);
        wb[t][1] = *reinterpret_cast<const bf16x8 *>(&sWb[16 * t + r16][32 + 8 * kg]);
    }
    constexpr int un_lim = UP * G;
    const int un_mine = r16 / G, g_mine = r16 - un_mine * G;     // image block (within a tile) of this lane's row
    // merged mode: the blocks' outputs are brought to a common maximum per query head and summed
    float gm = -INFINITY, sc[NT];
    if (p.merge) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int ul = 0; ul < UP; ++ul) gm = fmaxf(gm, sMx[16 * t + ul * G + g_mine]);
#pragma unroll
        for (int t = 0; t < NT; ++t) sc[t] = __expf(sMx[16 * t + r16] - gm);
    }
    f32x4 ysum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < NBATCH; ++kb) {
        const int un0 = kb * UBATCH;
        u32x4 (&cur)[UBATCH][2] = vfr[kb % (DEPTH + 1)];
        // (image blocks the workgroup does not have are clamped to its last one: no run-time test around loads)
        if (kb + DEPTH < NBATCH) load_values(un0 + DEPTH * UBATCH, vfr[(kb + DEPTH) % (DEPTH + 1)]);
        shift_tail(cur);
#pragma unroll
        for (int a = 0; a < UBATCH; ++a) {
            const int un = un0 + a;                      // image block within the workgroup
            const int t = un / UP, ul2 = un - t * UP;    // its MFMA tile and slot in the tile
            f32x4 o = {0.f, 0.f, 0.f, 0.f};
            o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cur[a][0]), wb[t][0], o, 0, 0, 0);
            o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cur[a][1]), wb[t][1], o, 0, 0, 0);
            const bool here = (present >> un) & 1ull;      // an absent block's values may be anything: selected away, never multiplied
            if (p.merge) {
                const bool mine = un_mine == ul2 && r16 < un_lim && here;          // rows of other blocks: cross terms
#pragma unroll
                for (int e = 0; e < 4; ++e) ysum[e] += mine ? sc[t] * o[e] : 0.f;
            } else if (un < nunits && un_mine == ul2 && r16 < un_lim) {
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = here ? o[e] : 0.f;
                const int ub = ub0 + un;
                const int b = quot(ub, p.qI), i = ub - b * p.I;
                float *yp = p.Ypart + (static_cast<size_t>(b * p.Hkv + h) * p.nparts + i * p.JS + s) * p.rec;
                *reinterpret_cast<f32x4 *>(yp + g_mine * D + 16 * wave + 4 * kg) = f32x4_mk(o[0], o[1], o[2], o[3]);
                if (wave == 0 && kg == 0) {
                    yp[G * D + g_mine] = sMx[16 * t + r16];
                    yp[G * D + G + g_mine] = s == 0 ? sSm[16 * t + r16] : 0.f;     // the block's mass is counted once
                }
            }
        }
    }
    if (p.merge) {
        // sum over the blocks of a tile: rows ul G + g for ul = 0 .. UP-1 sit in lanes of one 16-lane row
        if constexpr ((G & (G - 1)) == 0) {
#pragma unroll
            for (int o2 = G; o2 < 16; o2 <<= 1)
#pragma unroll
                for (int e = 0; e < 4; ++e) ysum[e] += __shfl_xor(ysum[e], o2, 64);
        } else {
            static_assert(UP == 2, "blocks of a tile are summed with one exchange");
#pragma unroll
            for (int e = 0; e < 4; ++e) ysum[e] += __shfl(ysum[e], (lane & 48) | ((r16 + G) & 15), 64);
        }
        if (r16 < G) {
            const int b = quot(ub0, p.qI), gi = (ub0 - b * p.I) / NU;
            float *yp = p.Ypart + (static_cast<size_t>(b * p.Hkv + h) * p.nparts + gi * p.JS + s) * p.rec;
            *reinterpret_cast<f32x4 *>(yp + r16 * D + 16 * wave + 4 * kg) = ysum;
            if (wave == 0 && kg == 0) {
                float sm = 0.f;
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int ul = 0; ul < UP; ++ul) sm += sSm[16 * t + ul * G + r16] * __expf(sMx[16 * t + ul * G + r16] - gm);
                yp[G * D + r16] = gm;
                yp[G * D + G + r16] = s == 0 ? sm : 0.f;                       // the blocks' mass is counted once
            }
        }
    }
    TS(2, 4);
}

// ------------------------------------------------------------------------------------------
// fd_finalize: joint softmax over all parts of one (batch, query head): rescale the partial
// outputs to the global maximum, normalise, add (sum P_vis) mu, store out and lse.
// ------------------------------------------------------------------------------------------
// PB = parts fetched per batch (a multiple of 8 covering all parts when there are at most 64).
template <int PB>
__global__ __launch_bounds__(128) void fd_finalize(Plan p, const uint16_t *__restrict__ mu,
                                                   uint16_t *__restrict__ out,
                                                   float *__restrict__ lse)
{
    // the arrival counters of fab_fused go back to zero
    if (p.fab && blockIdx.x == 0)
        for (int i = threadIdx.x; i < p.Hkv * p.NRB; i += 128) p.flags[static_cast<size_t>(i) * kCtrStride] = 0ull;
    KVC_FETCH_ARGS(p.B, lse, p.Ypart, p.qHkv, p.qG, p.nparts, p.rec, mu);
    __shared__ float sSc[kMaxParts + 64];
    __shared__ float sRed[2][3];
    TS(3, 0);
    // the head is the fast index of the workgroup id: ids are dealt round-robin over the XCDs, so a
    // head's rows are finished on the XCDs whose L2 saw its parts being written
    const int bgi = quot(blockIdx.x, p.qHkv), h = blockIdx.x - bgi * p.Hkv;
    const int b = quot(bgi, p.qG), g = bgi - b * p.G;
    const int bg = b * p.Hq + h * p.G + g;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rec = p.rec, GD = p.G * D;
    const float *yb = p.Ypart + static_cast<size_t>(b * p.Hkv + h) * p.nparts * rec;
    const int nvp = p.nvp;
    const int c = threadIdx.x;
    const float *yc = yb + g * D + c;
    // statistics first, then the first batch of partial outputs: one round trip for both
    float ml[2], sl[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int pt = min(static_cast<int>(threadIdx.x) + 128 * k, p.nparts - 1);
        ml[k] = yb[static_cast<size_t>(pt) * rec + GD + g];
        sl[k] = yb[static_cast<size_t>(pt) * rec + GD + p.G + g];
    }
    float v[PB];
#pragma unroll
    for (int k = 0; k < PB; ++k) v[k] = yc[static_cast<size_t>(min(k, p.nparts - 1)) * rec];
    TS(3, 1);
#pragma unroll
    for (int k = 0; k < 2; ++k)
        if (static_cast<int>(threadIdx.x) + 128 * k >= p.nparts) { ml[k] = -INFINITY; sl[k] = 0.f; }
    float mx = wave_max(fmaxf(ml[0], ml[1]));
    if (lane == 0) sRed[wave][0] = mx;
    if (threadIdx.x < 64) sSc[kMaxParts + threadIdx.x] = 0.f;
    __syncthreads();
    TS(3, 2);
    mx = fmaxf(sRed[0][0], sRed[1][0]);
    float a[2], z = 0.f, zv = 0.f;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int pt = threadIdx.x + 128 * k;
        a[k] = __expf(ml[k] - mx);              // exp(-inf) = 0 beyond the last part
        z += sl[k] * a[k];
        if (pt < nvp) zv += sl[k] * a[k];
    }
    z = wave_sum(z);
    zv = wave_sum(zv);
    if (lane == 0) { sRed[wave][1] = z; sRed[wave][2] = zv; }
    __syncthreads();
    z = sRed[0][1] + sRed[1][1];
    zv = sRed[0][2] + sRed[1][2];
    const float rz = 1.f / z;
#pragma unroll
    for (int k = 0; k < 2; ++k) sSc[threadIdx.x + 128 * k] = a[k] * rz;     // zero weight beyond the last part
    __syncthreads();
    TS(3, 3);
    float y = 0.f;
    for (int pt0 = 0; pt0 < p.nparts; pt0 += PB) {
        float cur[PB];
#pragma unroll
        for (int k = 0; k < PB; ++k) cur[k] = v[k];
        if (pt0 + PB < p.nparts) {
#pragma unroll
            for (int k = 0; k < PB; ++k) v[k] = yc[static_cast<size_t>(min(pt0 + PB + k, p.nparts - 1)) * rec];
        }
#pragma unroll
        for (int k = 0; k < PB; ++k) y += sSc[pt0 + k] * cur[k];    // clamped duplicates carry weight zero
    }
    y += (zv * rz) * bf_lo(mu[static_cast<size_t>(h) * D + c]);
    out[static_cast<size_t>(bg) * D + c] = f32_to_bf16_bits(y);
    if (c == 0 && lse) lse[bg] = mx + __logf(z);
    TS(3, 4);
}

// The same for at most 64 parts (PB = their number rounded up to eight): a lane per part holds its
// statistics, so each of the two waves finds the joint maximum and sum with shuffles alone -- no
// LDS, no barrier -- and all partial outputs are fetched in the same round trip as the statistics.
// What the kernel needs of the plan comes as 16 dwords of plain arguments: that many the hardware can
// hand to a wave in registers at its start (kernel-argument preload, see build.py), so that no
// memory round trip stands in front of the first loads.
template <int PB>
__global__ __launch_bounds__(128) void fd_finalize_few(const float *__restrict__ Ypart, const uint16_t *__restrict__ mu,
                                                       uint16_t *__restrict__ out, float *__restrict__ lse,
                                                       int a_Hkv, unsigned a_qHkv, int a_G, unsigned a_qG, int a_nparts,
                                                       int a_rec, int a_Hq, int a_nvp, u64 *a_flags, int a_nflags
#if defined(KVC_TIMELINE)
                                                       , unsigned long long *a_tl
#endif
                                                       )
{
    struct {
        int Hkv, G, Hq, nparts, rec, nvp;
        unsigned qHkv, qG;
        const float *Ypart;
#if defined(KVC_TIMELINE)
        unsigned long long *tl;
#endif
    } p = {a_Hkv, a_G, a_Hq, a_nparts, a_rec, a_nvp, a_qHkv, a_qG, Ypart
#if defined(KVC_TIMELINE)
           , a_tl
#endif
    };
    TS(3, 0);
    const int bgi = quot(blockIdx.x, p.qHkv), h = blockIdx.x - bgi * p.Hkv;
    const int b = quot(bgi, p.qG), g = bgi - b * p.G;
    const int bg = b * p.Hq + h * p.G + g;
    const int lane = threadIdx.x & 63, c = threadIdx.x;
    const int rec = p.rec, GD = p.G * D, np = p.nparts;
    const float *yb = p.Ypart + static_cast<size_t>(b * p.Hkv + h) * np * rec;
    const int pl = min(lane, np - 1);
    float ml = yb[static_cast<size_t>(pl) * rec + GD + g];
    float sl = yb[static_cast<size_t>(pl) * rec + GD + p.G + g];
    __builtin_amdgcn_sched_barrier(0);                   // the statistics are requested first: they are needed first
    const float *yc = yb + g * D + c;
    float v[PB];
#pragma unroll
    for (int k = 0; k < PB; ++k) v[k] = yc[static_cast<size_t>(min(k, np - 1)) * rec];
    const uint16_t mub = mu[static_cast<size_t>(h) * D + c];
    // all of the above is requested before anything is waited for (the instruction scheduler would move
    // part of the loads behind the reductions below: a second round trip)
    __builtin_amdgcn_sched_barrier(0);
    fetch_now(p.Hq, p.nvp);
    TS(3, 1);
    if (lane >= np) { ml = -INFINITY; sl = 0.f; }
    const float mx = wave_max(ml);
    const float a = __expf(ml - mx);                      // zero beyond the last part
    const float z = wave_sum(sl * a);
    const float zv = wave_sum(lane < p.nvp ? sl * a : 0.f);
    const float rz = 1.f / z;
    const float wgt = a * rz;
    TS(3, 3);
    float y = (zv * rz) * bf_lo(mub);
#pragma unroll
    for (int k = 0; k < PB; ++k) y += __shfl(wgt, k, 64) * v[k];     // clamped duplicates: weight zero
    out[static_cast<size_t>(bg) * D + c] = f32_to_bf16_bits(y);
    if (c == 0 && lse) lse[bg] = mx + __logf(z);
    // the arrival counters of fab_fused go back to zero
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < a_nflags; i += 128) a_flags[static_cast<size_t>(i) * kCtrStride] = 0ull;
    TS(3, 4);
}

size_t lds_b(int m_pad) { return static_cast<size_t>(kPC) * (m_pad + 8) * sizeof(uint16_t); }
size_t lds_c(int n, int nt)
{
    // rows of P, then one f32x4 per lane and tile for each of the four waves of k-half 1
    return static_cast<size_t>(16) * nt * (n + 8) * sizeof(uint16_t) + static_cast<size_t>(4) * nt * 64 * 16;
}

int units_per_group(int G)
{
    switch (G) {        // group sizes with a compiled kernel
    case 1: return 16;
    case 2: return 8;
    case 4: return 4;
    case 6: case 7: case 8: return 2;
    default: return 0;
    }
}

// padded: the query rows of whole image blocks fill 64-row blocks (what fab_fused needs); otherwise
// the rows are dense, r = (b I + i) G + g
Plan make_plan_layout(const kvc_shape &s, int t, int t_in, int cap, float scale, void *base, bool padded)
{
    Plan p;
    p.B = s.batch; p.Hq = s.n_q_heads; p.Hkv = s.n_kv_heads; p.G = p.Hq / p.Hkv;
    p.n = s.n_img_tokens; p.I = s.n_images; p.m = s.m;
    p.t = t; p.t_in = t_in; p.cap = cap; p.scale = scale;
    p.n_img = p.tlen = nullptr;
    {
        const int up = units_per_group(p.G), units = p.B * p.I;
        const int upb = up ? (64 / p.G) / (2 * up) * (2 * up) : 1;         // 64, 32, 16 or 8
        p.UPBs = 0;
        while ((1 << (p.UPBs + 1)) <= upb) ++p.UPBs;
        p.RV = (1 << p.UPBs) * p.G;
        if (!padded) { p.UPBs = kDenseRows; p.RV = 64; }                  // unit_row(ub) = ub G, every row valid
        p.R = units > 0 ? unit_row(units - 1, p.UPBs, p.G) + p.G : 0;
    }
    p.R_pad = static_cast<int>(align_up(p.R > 0 ? p.R : 1, kRB));
    // 64-row workgroups unless they would need more than two rounds over the CUs: then 128 rows per
    // workgroup re-read the theta chunk half as often
    p.RBW = (p.I > 0 && static_cast<long>((p.R + 63) / 64) * p.Hkv * (p.n / kPC) > 512) ? 8 : 4;
    p.NRB = p.I > 0 ? (p.R + 16 * p.RBW - 1) / (16 * p.RBW) : 0;       // row blocks that hold rows
    p.m_pad = static_cast<int>(align_up(p.m, 32));
    p.m16 = static_cast<int>(align_up(p.m, 16));
    p.NC = p.n / kPC;
    p.tiles_per_unit = p.m16 / 16;
    p.vis_tiles = p.B * p.Hkv * p.I * p.tiles_per_unit;
    p.nvis_a = (p.vis_tiles + 4 * kTPW - 1) / (4 * kTPW);
    p.UP = units_per_group(p.G);
    p.JS = (p.m + kJC - 1) / kJC;
    // two MFMA tiles of query rows per workgroup halve the re-streaming of U when the rows are there
    p.NT = (p.UP && p.B * p.I > p.UP) ? 2 : 1;
    // four tiles where the image blocks are short (n = 256: U and P are a large share of a workgroup's
    // bytes) and many: at least two workgroups per CU remain
    if (p.NT == 2 && p.n == 4 * kPC && !padded &&
        static_cast<long>((p.B * p.I + 4 * p.UP - 1) / (4 * p.UP)) * p.Hkv * p.JS >= 512)
        p.NT = 4;
    // developer knob (kvc_dev_decode_knobs): 1, 2 or 4 row tiles override the rule above
    if (g_force_nt && p.UP && p.B * p.I > p.UP) p.NT = g_force_nt == 1 ? 1 : (g_force_nt == 4 && p.n == 4 * kPC && !padded) ? 4 : 2;
    p.NG = p.UP ? (p.B * p.I + p.NT * p.UP - 1) / (p.NT * p.UP) : 0;
    p.NXC = (t + kXC - 1) / kXC;
    // the text chunks are extra workgroups of fc_fused; without vision tokens, of fa_scores
    p.ntext_a = (p.I > 0 && p.UP) ? 0 : p.B * p.Hkv * p.NXC;
    p.ntext_c = (p.I > 0 && p.UP) ? p.B * p.Hkv * p.NXC : 0;
    // When every workgroup of fc_fused holds image blocks of one batch element only, it merges them
    // into a single part record (fewer, larger-grained parts for fd_finalize to read)
    p.merge = (p.UP && p.I > 0 && p.I % (p.NT * p.UP) == 0) ? 1 : 0;
    p.nvp = (p.merge ? p.I / (p.NT * p.UP) : p.I) * p.JS;
    p.nparts = p.nvp + p.NXC;
    p.rec = static_cast<int>(align_up(p.G * D + 2 * p.G, 4));   // 16-byte aligned records
    p.nvis_b = static_cast<int>(align_up(p.NRB * p.Hkv, 8)) * p.NC;
    p.nvis_c = p.I > 0 ? static_cast<int>(align_up(p.NG * p.Hkv, 8)) * p.JS : 0;
    p.qNXC = quot_multiplier(p.NXC); p.qHkv = quot_multiplier(p.Hkv); p.qTPU = quot_multiplier(p.tiles_per_unit);
    p.qI = quot_multiplier(p.I); p.qNC = quot_multiplier(p.NC); p.qJS = quot_multiplier(p.JS); p.qG = quot_multiplier(p.G);

    const int nxc_max = (cap + kXC - 1) / kXC;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off += align_up(bytes, 256);
        return static_cast<char *>(base) + o;
    };
    p.flags = reinterpret_cast<u64 *>(take(static_cast<size_t>(kMaxFlags) * kCtrStride * sizeof(u64)));   // always first
    p.S = reinterpret_cast<uint16_t *>(take(static_cast<size_t>(p.Hkv) * p.R_pad * p.m_pad * 2));
    p.P = reinterpret_cast<uint16_t *>(take(static_cast<size_t>(p.Hkv) * p.R_pad * p.n * 2));
    p.stats = reinterpret_cast<f32x2 *>(take(static_cast<size_t>(p.Hkv) * p.R_pad * p.NC * 8));
    p.Ypart = reinterpret_cast<float *>(take(static_cast<size_t>(p.B) * p.Hkv * (p.I * p.JS + nxc_max) * p.rec * 4));
    p.fab = 0;
    p.wait_ticks = 0;
    p.epoch = 0;
    p.fallbacks = nullptr;
    p.bytes = off;
#if defined(KVC_TIMELINE)
    p.tl = nullptr;
#endif
    return p;
}

// fa_scores and fb_probs can run as one launch (fab_fused) when all its workgroups are resident at
// once (asked of the kernel instance, see fab_resident; never more than two per CU) and a
// workgroup's share of the score tiles is at most four per wave
bool fab_shape(const Plan &p)
{
    if (g_separate || p.I <= 0 || p.UPBs == kDenseRows) return false;
    const int T = p.tiles_per_unit * std::min(1 << p.UPBs, p.B * p.I), TW = (T + p.NC - 1) / p.NC;
    // (whether the chip holds all nvis_b workgroups at once is asked of the kernel instance: fab_resident)
    return p.RBW == 4 && p.nvis_b > 0 && p.nvis_b <= 512 && TW <= 16 && p.ntext_a == 0 && p.Hkv * p.NRB <= kMaxFlags;
}

// the padded row layout is used only where fab_fused can run; workspace sizes are taken from it
Plan make_plan(const kvc_shape &s, int t, int t_in, int cap, float scale, void *base, bool sizing = false)
{
    Plan p = make_plan_layout(s, t, t_in, cap, scale, base, true);
    if (!sizing && !fab_shape(p)) p = make_plan_layout(s, t, t_in, cap, scale, base, false);
    return p;
}

template <int PB> void launch_d1(const Plan &p, const DecodeCall &c)
{
    fd_finalize_few<PB><<<p.B * p.Hq, 128, 0, c.stream>>>(p.Ypart, static_cast<const uint16_t *>(c.mu),
                                                          static_cast<uint16_t *>(c.out), c.lse, p.Hkv, p.qHkv, p.G,
                                                          p.qG, p.nparts, p.rec, p.Hq, p.nvp, p.flags,
                                                          p.fab ? p.Hkv * p.NRB : 0
#if defined(KVC_TIMELINE)
                                                          , p.tl
#endif
                                                          );
}

void launch_d(const Plan &p, const DecodeCall &c)
{
    if (p.nparts > 64) {
        fd_finalize<64><<<p.B * p.Hq, 128, 0, c.stream>>>(p, static_cast<const uint16_t *>(c.mu),
                                                         static_cast<uint16_t *>(c.out), c.lse);
        return;
    }
    switch ((p.nparts + 7) >> 3) {      // parts, in eights
    case 1: launch_d1<8>(p, c); break;
    case 2: launch_d1<16>(p, c); break;
    case 3: launch_d1<24>(p, c); break;
    case 4: launch_d1<32>(p, c); break;
    case 5: launch_d1<40>(p, c); break;
    case 6: launch_d1<48>(p, c); break;
    case 7: launch_d1<56>(p, c); break;
    default: launch_d1<64>(p, c); break;
    }
}

template <int KS4, int NW> bool launch_b2(const Plan &p, const DecodeCall &c)
{
    static bool attr_set[kMaxDevices] = {};
    if (!allow_lds(reinterpret_cast<const void *>(fb_probs<KS4, NW>), kLdsBudget, attr_set)) return false;
    fb_probs<KS4, NW><<<p.nvis_b, 64 * NW, lds_b(p.m_pad), c.stream>>>(static_cast<const uint16_t *>(c.theta), p.S, p.qNC,
                                                                       p.NC, p.qHkv, p.Hkv, p.NRB, p.R, p.R_pad, p.m_pad,
                                                                       p.m, p.n, p);
    return true;
}

// ---- fab_fused: developer knobs and the debug counter --------------------------------------------------

static __device__ unsigned g_fab_fallbacks;          // workgroups that computed alone after a time-out

unsigned *fallback_counter()
{
    static std::mutex mu;
    static unsigned *ptr[kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *q = nullptr;
        if (hipGetSymbolAddress(&q, HIP_SYMBOL(g_fab_fallbacks)) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        ptr[dev] = static_cast<unsigned *>(q);
    }
    return ptr[dev];
}

// probe: no launch; true when all p.nvis_b workgroups of this instance can be resident at once (the
// capacity is taken for the largest LDS size of the instance and kept per device)
template <int KS4, int G> bool launch_ab3(const Plan &p, const DecodeCall &c, bool probe)
{
    static bool attr_set[kMaxDevices] = {};
    if (!allow_lds(reinterpret_cast<const void *>(fab_fused<KS4, G>), kLdsBudget, attr_set)) return false;
    if (probe) {
        static int capacity[kMaxDevices] = {};           // 0: not asked yet, -1: unknown
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
        if (capacity[dev] == 0) {
            int per_cu = 0, cus = 0;
            const bool ok = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fab_fused<KS4, G>, 256, lds_b(128 * KS4)) == hipSuccess &&
                            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess;
            capacity[dev] = (ok && per_cu > 0 && cus > 0) ? per_cu * cus : -1;
            if (!ok) (void)hipGetLastError();
        }
        return p.nvis_b <= capacity[dev];
    }
    fab_fused<KS4, G><<<p.nvis_b, 256, lds_b(p.m_pad), c.stream>>>(
        static_cast<const uint16_t *>(c.Kc), p.flags, p.qNC, p.NC, p.qHkv, p.Hkv, p.NRB * p.Hkv, p.tiles_per_unit, p.qTPU, p.UPBs,
        p.I, p.qI, p.m, p.B * p.I, p, static_cast<const uint16_t *>(c.theta), static_cast<const uint16_t *>(c.q));
    return true;
}

template <int KS4> bool launch_ab2(const Plan &p, const DecodeCall &c, bool probe)
{
    switch (p.G) {
    case 1: return launch_ab3<KS4, 1>(p, c, probe);
    case 2: return launch_ab3<KS4, 2>(p, c, probe);
    case 4: return launch_ab3<KS4, 4>(p, c, probe);
    case 6: return launch_ab3<KS4, 6>(p, c, probe);
    case 7: return launch_ab3<KS4, 7>(p, c, probe);
    default: return launch_ab3<KS4, 8>(p, c, probe);
    }
}

bool launch_ab(const Plan &p, const DecodeCall &c, bool probe = false)
{
    switch ((p.m_pad / 32 + 3) / 4) {
    case 1: return launch_ab2<1>(p, c, probe);
    case 2: return launch_ab2<2>(p, c, probe);
    case 3: return launch_ab2<3>(p, c, probe);
    case 4: return launch_ab2<4>(p, c, probe);
    case 5: return launch_ab2<5>(p, c, probe);
    case 6: return launch_ab2<6>(p, c, probe);
    case 7: return launch_ab2<7>(p, c, probe);
    case 8: return launch_ab2<8>(p, c, probe);
    default: return false;
    }
}

// fab_fused relies on all its workgroups being resident at once (its waiting workgroups would otherwise
// sit out their time limit and compute alone: correct, slow)
bool fab_resident(const Plan &p, const DecodeCall &c) { return launch_ab(p, c, true); }

template <int KS4> bool launch_b1(const Plan &p, const DecodeCall &c)
{
    return p.RBW == 8 ? launch_b2<KS4, 8>(p, c) : launch_b2<KS4, 4>(p, c);
}

bool launch_b(const Plan &p, const DecodeCall &c)
{
    switch ((p.m_pad / 32 + 3) / 4) {      // m <= n <= 1024: at most 8 groups of four k-steps
    case 1: return launch_b1<1>(p, c);
    case 2: return launch_b1<2>(p, c);
    case 3: return launch_b1<3>(p, c);
    case 4: return launch_b1<4>(p, c);
    case 5: return launch_b1<5>(p, c);
    case 6: return launch_b1<6>(p, c);
    case 7: return launch_b1<7>(p, c);
    case 8: return launch_b1<8>(p, c);
    default: return false;
    }
}

template <int G, bool TEXT, bool RAG> void launch_a2(const Plan &p, const DecodeCall &c, int grid)
{
    fa_scores<G, TEXT, RAG><<<grid, 256, 0, c.stream>>>(
        static_cast<const uint16_t *>(c.q), static_cast<const uint16_t *>(c.Kc), p.vis_tiles, p.qTPU,
        p.tiles_per_unit, p.qI, p.I, p.qHkv, p.Hkv, p.m, p.Hq, p.ntext_a, p,
        static_cast<uint16_t *>(c.Kt), static_cast<uint16_t *>(c.Vt),
        static_cast<const uint16_t *>(c.k_new), static_cast<const uint16_t *>(c.v_new));
}

template <int G> bool launch_a(const Plan &p, const DecodeCall &c)
{
    if (p.ntext_a + p.nvis_a == 0) return true;
    if (p.ntext_a > 0) {
        if (p.tlen) launch_a2<G, true, true>(p, c, p.ntext_a + p.nvis_a);
        else launch_a2<G, true, false>(p, c, p.ntext_a + p.nvis_a);
    } else {
        launch_a2<G, false, false>(p, c, p.nvis_a);
    }
    return true;
}

template <int G, int UP, int NT, int NC, bool RAG> bool launch_c4(const Plan &p, const DecodeCall &c)
{
    const size_t lds = std::max(lds_c(NC * kPC, NT), kTextLds);
    static bool attr_set[kMaxDevices] = {};
    if (!allow_lds(reinterpret_cast<const void *>(fc_fused<G, UP, NT, NC, RAG>), lds, attr_set)) return false;
    // U in the packed form where the caller has given it (only with whole blocks of 8 positions: n is a multiple of 64 here)
    const bool upk = c.U_packed != nullptr && g_use_packed_u;
    fc_fused<G, UP, NT, NC, RAG><<<p.nvis_c + p.ntext_c, 512, lds, c.stream>>>(
        static_cast<const uint16_t *>(upk ? c.U_packed : c.U), p.P, p.stats, p.qJS, p.JS, p.qHkv, p.Hkv, p.B, p.I, p.m,
        p.UPBs | (upk ? 256 : 0), p,
        static_cast<const uint16_t *>(c.Vc), static_cast<const uint16_t *>(c.q),
        static_cast<uint16_t *>(c.Kt), static_cast<uint16_t *>(c.Vt), static_cast<const uint16_t *>(c.k_new),
        static_cast<const uint16_t *>(c.v_new));
    return true;
}

template <int G, int UP, int NT, int NC> bool launch_c3(const Plan &p, const DecodeCall &c)
{
    return p.n_img ? launch_c4<G, UP, NT, NC, true>(p, c) : launch_c4<G, UP, NT, NC, false>(p, c);
}

template <int G, int UP, int NT> bool launch_c2(const Plan &p, const DecodeCall &c)
{
    switch (p.NC) {
    case 16: return launch_c3<G, UP, NT, 16>(p, c);
    case 9: return launch_c3<G, UP, NT, 9>(p, c);
    default: return launch_c3<G, UP, NT, 4>(p, c);
    }
}

template <int G, int UP> bool launch_ac(const Plan &p, const DecodeCall &c, bool first)
{
    if (first) return launch_a<G>(p, c);
    if (p.nvis_c == 0) return true;
    if (p.NT == 4) return launch_c3<G, UP, 4, 4>(p, c);     // compiled for n = 256 only
    return p.NT == 2 ? launch_c2<G, UP, 2>(p, c) : launch_c2<G, UP, 1>(p, c);
}

bool launch_for_group(const Plan &p, const DecodeCall &c, bool first)
{
    switch (p.G) {
    case 1: return launch_ac<1, 16>(p, c, first);
    case 2: return launch_ac<2, 8>(p, c, first);
    case 4: return launch_ac<4, 4>(p, c, first);
    case 6: return launch_ac<6, 2>(p, c, first);
    case 7: return launch_ac<7, 2>(p, c, first);
    default: return launch_ac<8, 2>(p, c, first);
    }
}

}  // namespace

// what the one-pass kernel shares with fab_fused: the call numbering, the waiting limit, the debug counter
unsigned next_decode_epoch()
{
    unsigned e = ++g_epoch;
    if (e == 0) e = ++g_epoch;                 // zero is what a finished call leaves behind
    return e;
}
int decode_wait_ticks() { return g_wait_ticks; }
unsigned *decode_fallback_counter() { return fallback_counter(); }

kvc_status finalize_parts(const float *Ypart, int nparts, int nvp, int rec, int B, int Hq, int Hkv, const void *mu,
                          void *out, float *lse, hipStream_t stream)
{
    if (nparts < 1 || nparts > 64) return KVC_ERR_UNSUPPORTED;
    Plan p;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.G = Hq / Hkv;
    p.qHkv = quot_multiplier(Hkv); p.qG = quot_multiplier(p.G);
    p.nparts = nparts; p.nvp = nvp; p.rec = rec;
    p.Ypart = const_cast<float *>(Ypart);
    p.flags = nullptr; p.fab = 0; p.NRB = 0;
#if defined(KVC_TIMELINE)
    p.tl = nullptr;
#endif
    DecodeCall c;
    c.mu = mu; c.out = out; c.lse = lse; c.stream = stream;
    launch_d(p, c);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_HIP;
}

void fast_decode_knobs(int row_tiles, int separate, int wait_ticks)
{
    if (row_tiles >= 0) g_force_nt = row_tiles;
    if (separate >= 0) g_separate = separate;
    if (wait_ticks >= 0) g_wait_ticks = wait_ticks;
}

// synchronous read of the debug counter (tests)
long fast_decode_fallbacks()
{
    unsigned *d = fallback_counter();
    unsigned v = 0;
    if (!d || hipMemcpy(&v, d, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess) return -1;
    return v;
}

bool fast_decode_supported(const kvc_shape &s)
{
    if (s.dtype != KVC_BF16 || s.head_dim != D) return false;
    if (units_per_group(s.n_q_heads / s.n_kv_heads) == 0) return false;
    // fc_fused is compiled for 4, 9 and 16 softmax tiles of 64 positions per image block
    if (s.n_img_tokens != 256 && s.n_img_tokens != 576 && s.n_img_tokens != 1024) return false;
    return lds_b(static_cast<int>(align_up(s.m, 32))) <= kLdsBudget;
}

size_t fast_decode_ws_bytes(const kvc_shape &s, int32_t max_text)
{
    return make_plan(s, max_text, max_text, max_text, 1.f, nullptr, true).bytes + kTimelineBytes;
}

kvc_status fast_decode(const DecodeCall &c)
{
    Plan p = make_plan(c.s, c.t, c.t_in, c.cap, c.scale, c.ws);
    if (p.nparts > kMaxParts) return generic_decode(c);
    // quot(): every dividend is a workgroup, tile or image-block index, every divisor one of these
    {
        const long args[] = {static_cast<long>(p.nvis_a) * 4 * kTPW, static_cast<long>(p.B) * p.Hkv * p.NXC, p.nvis_b, p.nvis_c,
                             static_cast<long>(p.B) * p.Hq, static_cast<long>(p.B) * p.Hkv * p.I + 64};
        const int divs[] = {p.NXC, p.Hkv, p.tiles_per_unit, p.I, p.NC, p.JS, p.G};
        long amax = 0, dmax = 1;
        for (long a : args) amax = a > amax ? a : amax;
        for (int d : divs) dmax = d > dmax ? d : dmax;
        if (amax * dmax >= (1ll << 32)) return generic_decode(c);
    }
    if (p.bytes > c.ws_bytes) return KVC_ERR_WORKSPACE;
    if (c.n_images_dev && c.text_len_dev) { p.n_img = c.n_images_dev; p.tlen = c.text_len_dev; }
#if defined(KVC_TIMELINE)
    p.tl = c.ws_bytes >= p.bytes + kTimelineBytes
               ? reinterpret_cast<unsigned long long *>(static_cast<char *>(c.ws) + ((c.ws_bytes - kTimelineBytes) & ~size_t(255)))
               : nullptr;
#endif
    if (fab_shape(p) && fab_resident(p, c)) {
        p.fab = 1;
        p.epoch = next_decode_epoch();
        p.wait_ticks = g_wait_ticks;
        p.fallbacks = fallback_counter();
    }
    if (p.fab) {
        if (!launch_ab(p, c)) return KVC_ERR_HIP;
    } else {
        if (!launch_for_group(p, c, true)) return KVC_ERR_HIP;
        if (p.nvis_b > 0) {
            if (!launch_b(p, c)) return KVC_ERR_HIP;
        }
    }
    if (!launch_for_group(p, c, false)) return KVC_ERR_HIP;
    launch_d(p, c);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_HIP;
}

}  // namespace kvc
