// Matrix-core decode path of KVCapsule for gfx950: bf16 storage, head_dim 128.
//
// One decode step of one layer = four launches that follow Alg. 1 of the paper
// (score-space order), with the softmax taken jointly over vision and text keys
// (Sec. 3.2) by carrying (max, sum) statistics per part and merging them at the end:
//
//   fa_scores   streams the compressed keys Kc and the text keys from HBM once:
//               S = sigma q Kc^T (Alg. 1 step 1) and the text logits, one 16x16x32 MFMA
//               tile per 16 key rows; also stores the new token's k, v in the text cache.
//   fb_probs    L = S theta (step 2) as a skinny GEMM per KV head, 64 query rows x 64
//               positions per workgroup with the theta chunk transposed into LDS on the way
//               in; emits P = exp(L - tile max) in bf16 and the tile's (max, sum) per row.
//   fc_fused    per (KV head, group of up to 16 query rows = whole image blocks, 64 rows j
//               of the capsule): W = sum_tiles alpha_tile (P_tile U_tile^T) with
//               alpha = exp(tile max - block max) (step 3; U streamed straight into MFMA
//               operands, P staged in LDS), then out_part = W Vc over the same 64 rows of
//               the compressed values (step 4; Vc's blocked layout is the MFMA operand),
//               un-normalised, with the block's (max, sum).  Text rows are handled by
//               trailing workgroups of the same launch (V_text transposed through LDS).
//   fd_finalize merges the parts of each (batch, query head) with the joint softmax
//               statistics, adds (sum P_vis) mu, writes out and lse.
//
// Only S and P (bf16), the tile statistics and the part records cross kernel boundaries;
// K_hat, V_hat and W never exist in memory.  Kernel boundaries are the only grid-wide synchronisation: a
// device-scope fence inside a kernel writes back and invalidates an XCD's whole L2 and costs
// far more than a launch.  Every kernel issues its independent loads in batches before the
// first use, because at these sizes the chain of dependent memory round trips, not bandwidth,
// sets the duration.
//
// Query rows of one KV head are ordered r = (b*I + i)*G + g, so the G query heads of a
// group and consecutive image blocks share MFMA tiles.
#include <stdlib.h>
#include "kvc_internal.h"

namespace kvc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;          // head_dim of this path
constexpr int kRB = 64;         // query rows per fb_probs workgroup (4 waves x 16)
constexpr int kPC = 64;         // positions per fb_probs workgroup (one softmax tile)
constexpr int kTPW = 2;         // 16-row key tiles per wavefront in fa_scores
constexpr int kJC = 64;         // capsule rows per fc_fused workgroup (one 16-row tile per wave)
constexpr int kXC = 128;        // text rows per fc_fused text workgroup
constexpr int kMaxN = 1024;     // fc_fused stages 16 rows of P (n bf16 each) in LDS
constexpr int kMaxParts = 256;  // fd_finalize keeps one scale per part in LDS
constexpr int kSWLD = kXC + 8;  // padded row (bf16) of the W tile / text probabilities in LDS
constexpr int kLDV = kXC + 8;   // padded row (bf16) of the transposed text values in LDS
constexpr size_t kLdsBudget = 150 * 1024;

struct Plan {
    int B, Hq, Hkv, G, n, I, m, t, t_in, cap;
    int R, R_pad, NRB, m_pad, m16, NC;
    int tiles_per_unit, vis_tiles, txt_tiles_per_bh, total_tiles;
    int ld_t;
    int UP, NG, JS, NXC, nparts, rec;
    int nvis_b, b_stride, nvis_c, c_stride;
    float scale;
    int dbg;
    unsigned long long *dbgbuf;
    uint16_t *S;
    uint16_t *P;
    float2 *stats;
    float *St;
    float *Ypart;
    size_t bytes;
};

// debug timestamps: kernel id, slot
#define TS(KID, K)                                                                        \
    do {                                                                                  \
        if (p.dbgbuf && threadIdx.x == 0)                                                 \
            p.dbgbuf[((KID) * 1024 + (blockIdx.x < 1024 ? blockIdx.x : 1023)) * 8 + (K)] = wall_clock64(); \
    } while (0)

__device__ inline bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ inline float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// ------------------------------------------------------------------------------------------
// fa_scores: Alg. 1 step 1 on the compressed keys, and the text logits.
// MFMA tile: A = 16 key rows x 32 channels, B = 32 channels x 16 query heads of the group,
// D[key row][head]; a lane ends up with 4 consecutive key rows of one head.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fa_scores(Plan p, const uint16_t *__restrict__ q,
                                                 const uint16_t *__restrict__ Kc,
                                                 uint16_t *__restrict__ Kt,
                                                 uint16_t *__restrict__ Vt,
                                                 const uint16_t *__restrict__ k_new,
                                                 const uint16_t *__restrict__ v_new)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, kg = lane >> 4;
    TS(0, 0);
    const int tile0 = (blockIdx.x * 4 + wave) * kTPW;
    uint4 kf[kTPW][4], qf[kTPW][4];
    bool live[kTPW];
#pragma unroll
    for (int tt = 0; tt < kTPW; ++tt) {
        const int tile = tile0 + tt;
        live[tt] = tile < p.total_tiles;
        if (!live[tt]) continue;
        const uint16_t *krow;
        int b, h;
        if (tile < p.vis_tiles) {
            const int u = tile / p.tiles_per_unit, jt = tile - u * p.tiles_per_unit;
            const int bh = u / p.I;
            b = bh / p.Hkv;
            h = bh - b * p.Hkv;
            const int row = min(jt * 16 + r16, p.m - 1);
            krow = Kc + (static_cast<size_t>(u) * p.m + row) * D;
        } else {
            const int tx = tile - p.vis_tiles;
            const int bh = tx / p.txt_tiles_per_bh, xt = tx - bh * p.txt_tiles_per_bh;
            b = bh / p.Hkv;
            h = bh - b * p.Hkv;
            const int x = min(xt * 16 + r16, p.t - 1);
            if (k_new && x == p.t_in) {
                // the new token: attend to it and store it in the text cache (Sec. 3.2)
                krow = k_new + static_cast<size_t>(bh) * D;
                const uint4 *ks = reinterpret_cast<const uint4 *>(krow) + kg;
                const uint4 *vs = reinterpret_cast<const uint4 *>(v_new + static_cast<size_t>(bh) * D) + kg;
                uint4 *kd = reinterpret_cast<uint4 *>(Kt + (static_cast<size_t>(bh) * p.cap + x) * D) + kg;
                uint4 *vd = reinterpret_cast<uint4 *>(Vt + (static_cast<size_t>(bh) * p.cap + x) * D) + kg;
                if (xt * 16 + r16 == x) {
#pragma unroll
                    for (int ks4 = 0; ks4 < 4; ++ks4) { kd[4 * ks4] = ks[4 * ks4]; vd[4 * ks4] = vs[4 * ks4]; }
                }
            } else {
                krow = Kt + (static_cast<size_t>(bh) * p.cap + x) * D;
            }
        }
        const uint4 *kp = reinterpret_cast<const uint4 *>(krow) + kg;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) kf[tt][ks] = kp[4 * ks];
        const int g = min(r16, p.G - 1);
        const uint4 *qp = reinterpret_cast<const uint4 *>(q + (static_cast<size_t>(b) * p.Hq + h * p.G + g) * D) + kg;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qf[tt][ks] = qp[4 * ks];
    }
    TS(0, 1);
#pragma unroll
    for (int tt = 0; tt < kTPW; ++tt) {
        if (!live[tt]) continue;
        const int tile = tile0 + tt;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kf[tt][ks]), as_bf16x8(qf[tt][ks]), acc, 0, 0, 0);
        if (r16 >= p.G) continue;      // columns beyond the group are copies of head G-1
        const int g = r16;
        if (tile < p.vis_tiles) {
            const int u = tile / p.tiles_per_unit, jt = tile - u * p.tiles_per_unit;
            const int bh = u / p.I, i = u - bh * p.I;
            const int b = bh / p.Hkv, h = bh - b * p.Hkv;
            const int r = (b * p.I + i) * p.G + g;
            const int j = jt * 16 + 4 * kg;
            uint32_t w[2];
#pragma unroll
            for (int e = 0; e < 4; e += 2) {
                const uint32_t lo = (j + e < p.m) ? f32_to_bf16_bits(acc[e] * p.scale) : 0u;
                const uint32_t hi = (j + e + 1 < p.m) ? f32_to_bf16_bits(acc[e + 1] * p.scale) : 0u;
                w[e >> 1] = lo | (hi << 16);
            }
            uint16_t *srow = p.S + (static_cast<size_t>(h) * p.R_pad + r) * p.m_pad + j;
            *reinterpret_cast<uint2 *>(srow) = make_uint2(w[0], w[1]);
            // the consumer reads whole 32-wide k-steps: keep the padding [m16, m_pad) at zero
            if (jt == p.tiles_per_unit - 1 && p.m_pad > p.m16) *reinterpret_cast<uint2 *>(srow + 16) = make_uint2(0u, 0u);
        } else {
            const int tx = tile - p.vis_tiles;
            const int bh = tx / p.txt_tiles_per_bh, xt = tx - bh * p.txt_tiles_per_bh;
            const int b = bh / p.Hkv, h = bh - b * p.Hkv;
            float4 o = make_float4(acc[0] * p.scale, acc[1] * p.scale, acc[2] * p.scale, acc[3] * p.scale);
            *reinterpret_cast<float4 *>(p.St + (static_cast<size_t>(b) * p.Hq + h * p.G + g) * p.ld_t + xt * 16 + 4 * kg) = o;
        }
    }
    TS(0, 4);
}


// ------------------------------------------------------------------------------------------
// fb_probs: Alg. 1 step 2 and the numerator of the softmax for one tile of 64 rows x 64
// positions: L[r][pos] = sum_j S[r][j] theta[j][pos], P = exp(L - tile max).
// MFMA tile: A = theta^T (16 positions x 32 j) from LDS, B = S^T (32 j x 16 rows) from
// memory, D[pos][row]: a lane ends up with 4 consecutive positions of one row.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fb_probs(Plan p, const uint16_t *__restrict__ theta)
{
    extern __shared__ __align__(16) uint16_t lds[];
    constexpr int PC = kPC;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, kg = lane >> 4;

    // rb is the slow index and its stride is a multiple of 8, so the workgroups that share a
    // (head, chunk) slice of theta land on the same XCD and share its L2
    const int rb = blockIdx.x / p.b_stride;
    const int hc = blockIdx.x - rb * p.b_stride;
    if (hc >= p.Hkv * p.NC) return;
    const int h = hc / p.NC, pc = hc - h * p.NC;

    TS(1, 0);
    const int LDT = p.m_pad + 8;
    uint16_t *ThT = lds;                 // [PC][LDT]   theta chunk, transposed: ThT[pos][j]

    // scores of this wave's 16 rows: first batch of fragments in flight during the LDS fill
    const int r0 = rb * kRB + wave * 16;
    const bool wave_live = r0 < p.R;
    const int r = r0 + r16;
    const uint16_t *srow = p.S + (static_cast<size_t>(h) * p.R_pad + r) * p.m_pad + 8 * kg;
    const int KS = p.m_pad / 32;
    constexpr int SB = 20;                       // m <= 640: every fragment in one batch
    uint4 sfr[SB];
#pragma unroll
    for (int k = 0; k < SB; ++k)
        sfr[k] = (wave_live && k < KS) ? *reinterpret_cast<const uint4 *>(srow + 32 * k) : make_uint4(0, 0, 0, 0);

    // ---- stage the theta chunk, transposed, in LDS -------------------------------------------------
    // a thread owns a pair of consecutive rows j, j+1 and 8 positions; the pair is packed so the
    // transposed store is one 32-bit word per position
    const int seg = (lane >> 4) + 4 * (wave & 1);          // 16-byte segment of the chunk row
    const int jp = (lane & 15) + 16 * (wave >> 1);         // row pair within a pass of 64 rows
    {
        const uint16_t *th = theta + static_cast<size_t>(h) * p.m * p.n + pc * PC + 8 * seg;
        constexpr int FB = 10;                   // passes per batch: m <= 640 is one batch
        for (int j0 = 2 * jp; j0 < p.m16; j0 += 64 * FB) {
            uint4 tv[FB][2];
#pragma unroll
            for (int k = 0; k < FB; ++k)
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int j = j0 + 64 * k + e;
                    tv[k][e] = make_uint4(0, 0, 0, 0);
                    if (j < p.m) tv[k][e] = *reinterpret_cast<const uint4 *>(th + static_cast<size_t>(j) * p.n);
                }
#pragma unroll
            for (int k = 0; k < FB; ++k) {
                const int j = j0 + 64 * k;
                if (j < p.m16) {
                    const uint32_t a[4] = {tv[k][0].x, tv[k][0].y, tv[k][0].z, tv[k][0].w};
                    const uint32_t c[4] = {tv[k][1].x, tv[k][1].y, tv[k][1].z, tv[k][1].w};
                    uint32_t *dst = reinterpret_cast<uint32_t *>(ThT + (8 * seg) * LDT + j);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        dst[(2 * e) * (LDT / 2)] = (a[e] & 0xffffu) | (c[e] << 16);
                        dst[(2 * e + 1) * (LDT / 2)] = (a[e] >> 16) | (c[e] & 0xffff0000u);
                    }
                }
            }
        }
        // zero the k padding of the transposed chunk: columns [m16, m_pad)
        const int padc = p.m_pad - p.m16;
        for (int idx = threadIdx.x; idx < PC * padc; idx += 256) {
            const int pp = idx / padc, j = p.m16 + idx - pp * padc;
            ThT[pp * LDT + j] = 0;
        }
    }
    __syncthreads();
    TS(1, 2);
    if (!wave_live) return;

    f32x4 acc[PC / 16];
#pragma unroll
    for (int mt = 0; mt < PC / 16; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int ks0 = 0; ks0 < KS; ks0 += SB) {
        uint4 cur[SB];
#pragma unroll
        for (int k = 0; k < SB; ++k) cur[k] = sfr[k];
#pragma unroll
        for (int k = 0; k < SB; ++k)
            if (ks0 + SB + k < KS) sfr[k] = *reinterpret_cast<const uint4 *>(srow + 32 * (ks0 + SB + k));
#pragma unroll
        for (int k = 0; k < SB; ++k) {
            const int ks = ks0 + k;
            if (ks < KS) {
                // scores beyond the compressed length are zeros written by fa_scores
                const bf16x8 bfrag = as_bf16x8(cur[k]);
#pragma unroll
                for (int mt = 0; mt < PC / 16; ++mt) {
                    const bf16x8 afrag = *reinterpret_cast<const bf16x8 *>(ThT + (16 * mt + r16) * LDT + 32 * ks + 8 * kg);
                    acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, bfrag, acc[mt], 0, 0, 0);
                }
            }
        }
    }

    TS(1, 3);
    // ---- tile-local softmax numerators of row r over the 64 positions ------------------------------
    float mx = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < PC / 16; ++mt)
#pragma unroll
        for (int e = 0; e < 4; ++e) mx = fmaxf(mx, acc[mt][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    float sum = 0.f;
    uint16_t *prow = p.P + (static_cast<size_t>(h) * p.R_pad + r) * p.n + pc * PC + 4 * kg;
#pragma unroll
    for (int mt = 0; mt < PC / 16; ++mt) {
        const uint32_t a0 = f32_to_bf16_bits(__expf(acc[mt][0] - mx)), a1 = f32_to_bf16_bits(__expf(acc[mt][1] - mx));
        const uint32_t a2 = f32_to_bf16_bits(__expf(acc[mt][2] - mx)), a3 = f32_to_bf16_bits(__expf(acc[mt][3] - mx));
        sum += __uint_as_float(a0 << 16) + __uint_as_float(a1 << 16) + __uint_as_float(a2 << 16) + __uint_as_float(a3 << 16);
        if (r < p.R) *reinterpret_cast<uint2 *>(prow + 16 * mt) = make_uint2(a0 | (a1 << 16), a2 | (a3 << 16));
    }
    sum += __shfl_xor(sum, 16, 64);
    sum += __shfl_xor(sum, 32, 64);
    if (kg == 0 && r < p.R) p.stats[(static_cast<size_t>(h) * p.R_pad + r) * p.NC + pc] = make_float2(mx, sum);
    TS(1, 4);
}

// ------------------------------------------------------------------------------------------
// fc_fused: Alg. 1 steps 3 and 4 on 64 rows of U / Vc for a group of query rows, and the
// text rows.  G query heads per KV head, UP image blocks per workgroup (G * UP <= 16 rows
// share the MFMA tile).
// Part record in Ypart: [G][D] floats of un-normalised output, [G] maxima, [G] sums.
// ------------------------------------------------------------------------------------------
template <int G, int UP>
__global__ __launch_bounds__(256) void fc_fused(Plan p, const uint16_t *__restrict__ U,
                                                const uint16_t *__restrict__ Vc,
                                                const uint16_t *__restrict__ Vt)
{
    static_assert(G * UP <= 16, "a row group must fit one MFMA tile");
    extern __shared__ __align__(16) uint16_t dyn[];      // vision: P [16][n + 8]; text: V^T [D][kLDV]
    __shared__ __align__(16) uint16_t sWb[16][kSWLD];    // W tile / text probabilities, bf16
    __shared__ float sAl[16][17];                        // alpha[row][tile]
    __shared__ float sMx[16], sSm[16];
    __shared__ float sRed[4][16][2];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, kg = lane >> 4;
    const int rec = p.rec;

    if (static_cast<int>(blockIdx.x) >= p.nvis_c) {
        // ---------------- text rows: one chunk of kXC rows of one (batch, KV head) ----------------
        TS(2, 0);
        const int id = blockIdx.x - p.nvis_c;
        const int bh = id / p.NXC, xc = id - bh * p.NXC;
        const int b = bh / p.Hkv, h = bh - b * p.Hkv;
        const int lo = xc * kXC, hi = min(p.t, lo + kXC);
        // value rows -> LDS transposed: sVt[c][x]
        {
            const int rowl = wave * 4 + kg, cs = r16;
            const uint4 *sp = reinterpret_cast<const uint4 *>(Vt + static_cast<size_t>(bh) * p.cap * D) + cs;
            uint4 vb[kXC / 16];
#pragma unroll
            for (int it = 0; it < kXC / 16; ++it) vb[it] = sp[static_cast<size_t>(min(lo + rowl + 16 * it, hi - 1)) * (D / 8)];
#pragma unroll
            for (int it = 0; it < kXC / 16; ++it) {
                const uint32_t w4[4] = {vb[it].x, vb[it].y, vb[it].z, vb[it].w};
                uint16_t *dst = dyn + (8 * cs) * kLDV + rowl + 16 * it;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    dst[(2 * e) * kLDV] = static_cast<uint16_t>(w4[e] & 0xffffu);
                    dst[(2 * e + 1) * kLDV] = static_cast<uint16_t>(w4[e] >> 16);
                }
            }
        }
        // probabilities relative to the chunk's own maximum: LPR lanes per row
        constexpr int LPR = 256 / kXC, NG = (G + LPR - 1) / LPR;
        const int xl = threadIdx.x / LPR, x = lo + xl, gsub = threadIdx.x % LPR;
        float sc[NG];
#pragma unroll
        for (int k = 0; k < NG; ++k) {
            const int g = gsub + LPR * k;
            sc[k] = (g < G && x < hi) ? p.St[(static_cast<size_t>(b) * p.Hq + h * G + g) * p.ld_t + x] : -INFINITY;
        }
#pragma unroll
        for (int k = 0; k < NG; ++k) {
            float mx = sc[k];                       // max over rows = lanes with equal (lane % LPR)
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
            if (lane < LPR && lane + LPR * k < G) sRed[wave][lane + LPR * k][0] = mx;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < NG; ++k) {
            const int g = gsub + LPR * k;
            float e = 0.f, mx = 0.f;
            if (g < G) {
                mx = fmaxf(fmaxf(sRed[0][g][0], sRed[1][g][0]), fmaxf(sRed[2][g][0], sRed[3][g][0]));
                const uint32_t eb = x < hi ? f32_to_bf16_bits(__expf(sc[k] - mx)) : 0u;
                e = __uint_as_float(eb << 16);
                sWb[g][xl] = static_cast<uint16_t>(eb);
            }
            float sm = e;
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) sm += __shfl_xor(sm, o, 64);
            if (lane < LPR && g < G) sRed[wave][g][1] = sm;
            if (threadIdx.x < LPR && g < G) sMx[g] = mx;
        }
        for (int idx = threadIdx.x; idx < (16 - G) * kXC; idx += 256) sWb[G + idx / kXC][idx % kXC] = 0;
        __syncthreads();
        // out_part^T[c][g] = sum_x V^T[c][x] P[g][x]; each wave owns two 16-channel tiles
        float *yp = p.Ypart + (static_cast<size_t>(bh) * p.nparts + p.I * p.JS + xc) * rec;
#pragma unroll
        for (int ct2 = 0; ct2 < 2; ++ct2) {
            const int ct = 2 * wave + ct2;
            f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < kXC / 32; ++ks) {
                const bf16x8 afrag = *reinterpret_cast<const bf16x8 *>(dyn + (16 * ct + r16) * kLDV + 32 * ks + 8 * kg);
                const bf16x8 bfrag = *reinterpret_cast<const bf16x8 *>(&sWb[r16][32 * ks + 8 * kg]);
                o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, bfrag, o, 0, 0, 0);
            }
            if (r16 < G) *reinterpret_cast<float4 *>(yp + r16 * D + 16 * ct + 4 * kg) = make_float4(o[0], o[1], o[2], o[3]);
        }
        if (threadIdx.x < G) {
            yp[G * D + threadIdx.x] = sMx[threadIdx.x];
            yp[G * D + G + threadIdx.x] = sRed[0][threadIdx.x][1] + sRed[1][threadIdx.x][1] +
                                          sRed[2][threadIdx.x][1] + sRed[3][threadIdx.x][1];
        }
        TS(2, 4);
        return;
    }

    // ---------------- vision: (row group ug, KV head h, slice s of the capsule rows) ----------------
    // ug is the slow index with a stride that is a multiple of 8: workgroups that stream the same
    // rows of U[h] sit on one XCD and share its L2
    TS(2, 0);
    const int ug = blockIdx.x / p.c_stride;
    const int hs = blockIdx.x - ug * p.c_stride;
    if (hs >= p.Hkv * p.JS) return;
    const int h = hs / p.JS, s = hs - h * p.JS;
    const int ub0 = ug * UP;
    const int nunits = min(UP, p.B * p.I - ub0);
    const int nrows = nunits * G, r0 = ub0 * G;
    const int lo = s * kJC, hi = min(p.m, lo + kJC);
    const int n = p.n, LDP = n + 8, NC = p.NC;
    uint16_t *sP = dyn;

    // ---- everything this workgroup reads is requested up front ------------------------------------------
    // U rows of this wave's 16-row tile, first batch of MFMA operands
    const bool tile_live = lo + 16 * wave < hi;
    const uint16_t *urow = U + (static_cast<size_t>(h) * p.m + min(lo + 16 * wave + r16, p.m - 1)) * n + 8 * kg;
    const int KS = n / 32;
    constexpr int UBK = 8;
    uint4 ufr[UBK];
#pragma unroll
    for (int k = 0; k < UBK; ++k)
        ufr[k] = (tile_live && k < KS) ? *reinterpret_cast<const uint4 *>(urow + 32 * k) : make_uint4(0, 0, 0, 0);
    // P rows of the group -> LDS (16 threads per row, 16 bytes each per pass)
    uint4 pfr[kMaxN / 128];
    {
        const int row = threadIdx.x >> 4, sub = threadIdx.x & 15;
        const uint4 *prow = reinterpret_cast<const uint4 *>(p.P + (static_cast<size_t>(h) * p.R_pad + r0 + min(row, nrows - 1)) * n) + sub;
#pragma unroll
        for (int k = 0; k < kMaxN / 128; ++k)
            pfr[k] = (16 * k + sub < n / 8 && row < nrows) ? prow[16 * k] : make_uint4(0, 0, 0, 0);
    }
    // tile statistics of row (lane & 15): one float2 per tile, lanes with kg > 0 idle
    float2 st[kMaxN / kPC];
    {
        const float2 *sp = p.stats + (static_cast<size_t>(h) * p.R_pad + r0 + min(r16, nrows - 1)) * NC;
#pragma unroll
        for (int k = 0; k < kMaxN / kPC; ++k) st[k] = (wave == 0 && kg == 0 && k < NC) ? sp[k] : make_float2(-INFINITY, 0.f);
    }
    // compressed values: wave w owns channel tiles 2w, 2w+1; the operand (8 rows j of one
    // channel) is 16 contiguous bytes in the blocked layout.  Blocks of the group are handled in
    // batches of UBATCH; the first batch is requested here.
    constexpr int UBATCH = UP < 4 ? UP : 4;
    const int jb0 = lo / 8;
    // a shorter last block ([D][w], w = m % 8) exists only in the last slice: uniform branch
    const bool has_tail = (p.m & 7) != 0 && hi == p.m;
    auto load_values = [&](int un0, uint4 (&dst)[UBATCH][2][2]) {
#pragma unroll
        for (int a = 0; a < UBATCH; ++a) {
            const int ub = ub0 + min(un0 + a, nunits - 1);
            const int b = ub / p.I, i = ub - b * p.I;
            const uint16_t *vbase = Vc + (static_cast<size_t>(b * p.Hkv + h) * p.I + i) * p.m * D;
#pragma unroll
            for (int ct2 = 0; ct2 < 2; ++ct2)
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    const int jb = jb0 + 4 * ks + kg, c = 16 * (2 * wave + ct2) + r16;
                    dst[a][ct2][ks] = (8 * jb + 8 <= p.m)
                                          ? *reinterpret_cast<const uint4 *>(vbase + static_cast<size_t>(jb) * 8 * D + c * 8)
                                          : make_uint4(0, 0, 0, 0);
                }
            if (has_tail) {
#pragma unroll
                for (int ct2 = 0; ct2 < 2; ++ct2)
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        const int jb = jb0 + 4 * ks + kg, c = 16 * (2 * wave + ct2) + r16;
                        if (8 * jb < p.m && 8 * jb + 8 > p.m) {
                            const int w = p.m - 8 * jb;
                            const uint16_t *tp = vbase + static_cast<size_t>(jb) * 8 * D + c * w;
                            uint32_t e[8];
#pragma unroll
                            for (int q2 = 0; q2 < 8; ++q2) e[q2] = q2 < w ? tp[q2] : 0u;
                            dst[a][ct2][ks] = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
                        }
                    }
            }
        }
    };
    uint4 vfr[UBATCH][2][2];
    load_values(0, vfr);

    TS(2, 1);
    // ---- block statistics: alpha[row][tile] = exp(tile max - block max) ----------------------------------
    if (wave == 0 && kg == 0) {
        float mx = -INFINITY;
#pragma unroll
        for (int k = 0; k < kMaxN / kPC; ++k) mx = fmaxf(mx, st[k].x);
        float sm = 0.f;
#pragma unroll
        for (int k = 0; k < kMaxN / kPC; ++k) {
            const float a = k < NC ? __expf(st[k].x - mx) : 0.f;
            sm += st[k].y * a;
            sAl[r16][k] = a;
        }
        sMx[r16] = mx;
        sSm[r16] = sm;
    }
    {
        const int row = threadIdx.x >> 4, sub = threadIdx.x & 15;
        uint4 *dst = reinterpret_cast<uint4 *>(sP + row * LDP) + sub;
#pragma unroll
        for (int k = 0; k < kMaxN / 128; ++k)
            if (16 * k + sub < n / 8) dst[16 * k] = pfr[k];
    }
    __syncthreads();
    TS(2, 2);

    // ---- step 3: W^T[j][row] = sum_tiles alpha[row][tile] sum_pos U[j][pos] P[row][pos] ------------------
    {
        f32x4 w = {0.f, 0.f, 0.f, 0.f};
        if (tile_live) {
            const uint16_t *pb = sP + r16 * LDP + 8 * kg;
            for (int ks0 = 0; ks0 < KS; ks0 += UBK) {
                uint4 cur[UBK];
#pragma unroll
                for (int k = 0; k < UBK; ++k) cur[k] = ufr[k];
#pragma unroll
                for (int k = 0; k < UBK; ++k)
                    if (ks0 + UBK + k < KS) ufr[k] = *reinterpret_cast<const uint4 *>(urow + 32 * (ks0 + UBK + k));
#pragma unroll
                for (int k = 0; k < UBK; k += 2) {
                    if (ks0 + k < KS) {            // one softmax tile = 64 positions = two k-steps
                        f32x4 wt = {0.f, 0.f, 0.f, 0.f};
                        wt = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            as_bf16x8(cur[k]), *reinterpret_cast<const bf16x8 *>(pb + 32 * (ks0 + k)), wt, 0, 0, 0);
                        wt = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            as_bf16x8(cur[k + 1]), *reinterpret_cast<const bf16x8 *>(pb + 32 * (ks0 + k + 1)), wt, 0, 0, 0);
                        const float al = sAl[r16][(ks0 + k) >> 1];
                        w[0] += al * wt[0]; w[1] += al * wt[1]; w[2] += al * wt[2]; w[3] += al * wt[3];
                    }
                }
            }
        }
        const int jl = 16 * wave + 4 * kg;
        const uint32_t w0 = (lo + jl + 0 < hi) ? f32_to_bf16_bits(w[0]) : 0u, w1 = (lo + jl + 1 < hi) ? f32_to_bf16_bits(w[1]) : 0u;
        const uint32_t w2 = (lo + jl + 2 < hi) ? f32_to_bf16_bits(w[2]) : 0u, w3 = (lo + jl + 3 < hi) ? f32_to_bf16_bits(w[3]) : 0u;
        *reinterpret_cast<uint2 *>(&sWb[r16][jl]) = make_uint2(w0 | (w1 << 16), w2 | (w3 << 16));
    }
    __syncthreads();
    TS(2, 3);

    // ---- step 4: out_part^T[c][row] = sum_j Vc^T[c][j] W[row][j], per image block of the group -----------
    const bf16x8 wb0 = *reinterpret_cast<const bf16x8 *>(&sWb[r16][8 * kg]);
    const bf16x8 wb1 = *reinterpret_cast<const bf16x8 *>(&sWb[r16][32 + 8 * kg]);
    const int un_mine = r16 / G, g_mine = r16 - un_mine * G;
#pragma unroll
    for (int un0 = 0; un0 < UP; un0 += UBATCH) {
        uint4 cur[UBATCH][2][2];
#pragma unroll
        for (int a = 0; a < UBATCH; ++a)
#pragma unroll
            for (int ct2 = 0; ct2 < 2; ++ct2)
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) cur[a][ct2][ks] = vfr[a][ct2][ks];
        if (un0 + UBATCH < UP && un0 + UBATCH < nunits) load_values(un0 + UBATCH, vfr);
#pragma unroll
        for (int a = 0; a < UBATCH; ++a) {
            const int un = un0 + a;
            const int ub = ub0 + un;
            const int b = ub / p.I, i = ub - b * p.I;
            float *yp = p.Ypart + (static_cast<size_t>(b * p.Hkv + h) * p.nparts + i * p.JS + s) * rec;
            const bool mine = un < nunits && un_mine == un && r16 < nrows;
#pragma unroll
            for (int ct2 = 0; ct2 < 2; ++ct2) {
                f32x4 o = {0.f, 0.f, 0.f, 0.f};
                o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cur[a][ct2][0]), wb0, o, 0, 0, 0);
                o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cur[a][ct2][1]), wb1, o, 0, 0, 0);
                if (mine)
                    *reinterpret_cast<float4 *>(yp + g_mine * D + 16 * (2 * wave + ct2) + 4 * kg) = make_float4(o[0], o[1], o[2], o[3]);
            }
            if (wave == 0 && kg == 0 && mine) {
                yp[G * D + g_mine] = sMx[r16];
                yp[G * D + G + g_mine] = s == 0 ? sSm[r16] : 0.f;     // the block's mass is counted once
            }
        }
    }
    TS(2, 4);
}

// ------------------------------------------------------------------------------------------
// fd_finalize: joint softmax over all parts of one (batch, query head): rescale the partial
// outputs to the global maximum, normalise, add (sum P_vis) mu, store out and lse.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(128) void fd_finalize(Plan p, const uint16_t *__restrict__ mu,
                                                   uint16_t *__restrict__ out,
                                                   float *__restrict__ lse)
{
    __shared__ float sSc[kMaxParts];
    __shared__ float sRed[2][3];
    TS(3, 0);
    const int bg = blockIdx.x, b = bg / p.Hq, gq = bg - b * p.Hq;
    const int h = gq / p.G, g = gq - h * p.G;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rec = p.rec, GD = p.G * D;
    const float *yb = p.Ypart + static_cast<size_t>(b * p.Hkv + h) * p.nparts * rec;
    const int nvp = p.I * p.JS;
    const int c = threadIdx.x;
    const float *yc = yb + g * D + c;
    // first batch of partial outputs in flight together with the statistics
    constexpr int PB = 64;
    float v[PB];
#pragma unroll
    for (int k = 0; k < PB; ++k) v[k] = yc[static_cast<size_t>(min(k, p.nparts - 1)) * rec];
    float ml[2], sl[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int pt = threadIdx.x + 128 * k;
        ml[k] = pt < p.nparts ? yb[static_cast<size_t>(pt) * rec + GD + g] : -INFINITY;
        sl[k] = pt < p.nparts ? yb[static_cast<size_t>(pt) * rec + GD + p.G + g] : 0.f;
    }
    float mx = wave_max(fmaxf(ml[0], ml[1]));
    if (lane == 0) sRed[wave][0] = mx;
    __syncthreads();
    mx = fmaxf(sRed[0][0], sRed[1][0]);
    float a[2], z = 0.f, zv = 0.f;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int pt = threadIdx.x + 128 * k;
        a[k] = pt < p.nparts ? __expf(ml[k] - mx) : 0.f;
        z += sl[k] * a[k];
        if (pt < nvp) zv += sl[k] * a[k];
    }
    z = wave_sum(z);
    zv = wave_sum(zv);
    if (lane == 0) { sRed[wave][1] = z; sRed[wave][2] = zv; }
    __syncthreads();
    z = sRed[0][1] + sRed[1][1];
    zv = sRed[0][2] + sRed[1][2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int pt = threadIdx.x + 128 * k;
        if (pt < p.nparts) sSc[pt] = a[k] / z;
    }
    __syncthreads();
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
        for (int k = 0; k < PB; ++k)
            if (pt0 + k < p.nparts) y += sSc[pt0 + k] * cur[k];
    }
    y += (zv / z) * bf_lo(mu[static_cast<size_t>(h) * D + c]);
    out[static_cast<size_t>(bg) * D + c] = f32_to_bf16_bits(y);
    if (c == 0 && lse) lse[bg] = mx + __logf(z);
    TS(3, 4);
}

size_t lds_b(int m_pad) { return static_cast<size_t>(kPC) * (m_pad + 8) * sizeof(uint16_t); }
size_t lds_c(int n)
{
    const size_t vis = static_cast<size_t>(16) * (n + 8) * sizeof(uint16_t);
    const size_t txt = static_cast<size_t>(D) * kLDV * sizeof(uint16_t);
    return vis > txt ? vis : txt;
}

int units_per_group(int G)
{
    switch (G) {
    case 1: return 16;
    case 2: return 8;
    case 4: return 4;
    case 7: case 8: return 2;
    case 16: return 1;
    default: return 0;
    }
}

Plan make_plan(const kvc_shape &s, int t, int t_in, int cap, float scale, void *base)
{
    Plan p;
    p.B = s.batch; p.Hq = s.n_q_heads; p.Hkv = s.n_kv_heads; p.G = p.Hq / p.Hkv;
    p.n = s.n_img_tokens; p.I = s.n_images; p.m = s.m;
    p.t = t; p.t_in = t_in; p.cap = cap; p.scale = scale;
    { const char *e = getenv("KVC_DBG"); p.dbg = e ? atoi(e) : 0; }
    p.R = p.B * p.I * p.G;
    p.R_pad = static_cast<int>(align_up(p.R > 0 ? p.R : 1, kRB));
    p.NRB = p.I > 0 ? p.R_pad / kRB : 0;
    p.m_pad = static_cast<int>(align_up(p.m, 32));
    p.m16 = static_cast<int>(align_up(p.m, 16));
    p.NC = p.n / kPC;
    p.tiles_per_unit = p.m16 / 16;
    p.vis_tiles = p.B * p.Hkv * p.I * p.tiles_per_unit;
    p.txt_tiles_per_bh = (t + 15) / 16;
    p.total_tiles = p.vis_tiles + p.B * p.Hkv * p.txt_tiles_per_bh;
    p.ld_t = static_cast<int>(align_up(cap > 0 ? cap : 1, 16));
    p.UP = units_per_group(p.G);
    p.NG = p.UP ? (p.B * p.I + p.UP - 1) / p.UP : 0;
    p.JS = (p.m + kJC - 1) / kJC;
    p.NXC = (t + kXC - 1) / kXC;
    p.nparts = p.I * p.JS + p.NXC;
    p.rec = static_cast<int>(align_up(p.G * D + 2 * p.G, 4));   // 16-byte aligned records
    p.b_stride = static_cast<int>(align_up(p.Hkv * p.NC, 8));
    p.nvis_b = p.NRB * p.b_stride;
    p.c_stride = static_cast<int>(align_up(p.Hkv * p.JS, 8));
    p.nvis_c = p.I > 0 ? p.NG * p.c_stride : 0;

    const int nxc_max = (cap + kXC - 1) / kXC;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off += align_up(bytes, 256);
        return static_cast<char *>(base) + o;
    };
    p.S = reinterpret_cast<uint16_t *>(take(static_cast<size_t>(p.Hkv) * p.R_pad * p.m_pad * 2));
    p.P = reinterpret_cast<uint16_t *>(take(static_cast<size_t>(p.Hkv) * p.R_pad * p.n * 2));
    p.stats = reinterpret_cast<float2 *>(take(static_cast<size_t>(p.Hkv) * p.R_pad * p.NC * 8));
    p.St = reinterpret_cast<float *>(take(static_cast<size_t>(p.B) * p.Hq * p.ld_t * 4));
    p.Ypart = reinterpret_cast<float *>(take(static_cast<size_t>(p.B) * p.Hkv * (p.I * p.JS + nxc_max) * p.rec * 4));
    p.bytes = off;
    p.dbgbuf = nullptr;
    return p;
}

template <int G, int UP> kvc_status launch_c(const Plan &p, const DecodeCall &c)
{
    const int grid = p.nvis_c + p.B * p.Hkv * p.NXC;
    fc_fused<G, UP><<<grid, 256, lds_c(p.n), c.stream>>>(p, static_cast<const uint16_t *>(c.U),
                                                         static_cast<const uint16_t *>(c.Vc),
                                                         static_cast<const uint16_t *>(c.Vt));
    return KVC_OK;
}

}  // namespace

bool fast_decode_supported(const kvc_shape &s)
{
    if (s.dtype != KVC_BF16 || s.head_dim != D) return false;
    if (units_per_group(s.n_q_heads / s.n_kv_heads) == 0) return false;
    if (s.n_img_tokens % kPC != 0 || s.n_img_tokens > kMaxN) return false;
    return lds_b(static_cast<int>(align_up(s.m, 32))) <= kLdsBudget;
}

size_t fast_decode_ws_bytes(const kvc_shape &s, int32_t max_text)
{
    return make_plan(s, max_text, max_text, max_text, 1.f, nullptr).bytes;
}

kvc_status fast_decode(const DecodeCall &c)
{
    Plan p = make_plan(c.s, c.t, c.t_in, c.cap, c.scale, c.ws);
    if (p.nparts > kMaxParts) return generic_decode(c);
    if (p.bytes > c.ws_bytes) return KVC_ERR_WORKSPACE;
    p.dbgbuf = (p.dbg & 256) && c.ws_bytes >= p.bytes + (1 << 20)
                   ? reinterpret_cast<unsigned long long *>(static_cast<char *>(c.ws) + ((c.ws_bytes - (1 << 20)) & ~size_t(255)))
                   : nullptr;
    const int waves = (p.total_tiles + kTPW - 1) / kTPW;
    fa_scores<<<(waves + 3) / 4, 256, 0, c.stream>>>(
        p, static_cast<const uint16_t *>(c.q), static_cast<const uint16_t *>(c.Kc),
        static_cast<uint16_t *>(c.Kt), static_cast<uint16_t *>(c.Vt),
        static_cast<const uint16_t *>(c.k_new), static_cast<const uint16_t *>(c.v_new));
    if (p.nvis_b > 0) {
        static bool attr_set = false;
        if (!attr_set) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(fb_probs),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    static_cast<int>(kLdsBudget)) != hipSuccess)
                return KVC_ERR_HIP;
            attr_set = true;
        }
        fb_probs<<<p.nvis_b, 256, lds_b(p.m_pad), c.stream>>>(p, static_cast<const uint16_t *>(c.theta));
    }
    kvc_status st;
    switch (p.G) {
    case 1: st = launch_c<1, 16>(p, c); break;
    case 2: st = launch_c<2, 8>(p, c); break;
    case 4: st = launch_c<4, 4>(p, c); break;
    case 7: st = launch_c<7, 2>(p, c); break;
    case 8: st = launch_c<8, 2>(p, c); break;
    default: st = launch_c<16, 1>(p, c); break;
    }
    if (st != KVC_OK) return st;
    fd_finalize<<<p.B * p.Hq, 128, 0, c.stream>>>(p, static_cast<const uint16_t *>(c.mu),
                                                  static_cast<uint16_t *>(c.out), c.lse);
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_HIP;
}

}  // namespace kvc
