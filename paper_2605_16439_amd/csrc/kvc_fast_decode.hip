// Matrix-core decode path of KVCapsule for gfx950: bf16 storage, head_dim 128.
//
// One decode step of one layer = four launches that follow Alg. 1 of the paper
// (score-space order), with the softmax taken jointly over vision and text keys
// (Sec. 3.2) by carrying (max, sum) statistics per tile and merging them at the end:
//
//   fa_scores   streams the compressed keys Kc and the text keys from HBM once,
//               S = sigma q Kc^T (Alg. 1 step 1) and the text logits, one 16x16x32 MFMA
//               tile per 16 key rows; also stores the new token's k, v in the text cache.
//   fb_expand   per (KV head, 64 query rows, chunk of PC positions of an image block):
//               L = S theta (step 2), P = exp(L - tile max), W_part = P U^T (step 3).  theta
//               and U chunks are staged in LDS (theta transposed on the way in) and shared
//               by the four wavefronts; the P tile goes from the accumulator layout of the
//               first MFMA straight into the operand layout of the second.
//   fc_output   streams the compressed values Vc and the text values once (step 4 and the
//               text part): each workgroup merges the chunk partials of W for its rows and
//               emits an un-normalised partial output with its own (max, sum).
//   fd_finalize merges the partial outputs of each (batch, KV head) with the joint softmax
//               statistics, adds (sum P_vis) mu, writes out and lse.
// Kernel boundaries are the only grid-wide synchronisation: device-scope fences inside a
// kernel write back and invalidate the L2 of an XCD and cost far more than a launch.
//
// Query rows of one KV head are ordered r = (b*I + i)*G + g, so the G query heads of a
// group and all image blocks of a batch element share MFMA tiles.
#include "kvc_internal.h"

namespace kvc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;          // head_dim of this path
constexpr int kRB = 64;         // query rows per fb_expand workgroup (4 waves x 16)
constexpr int kTPW = 2;         // 16-row key tiles per wavefront in fa_scores
constexpr int kXC = 128;        // text rows per fc_output workgroup
constexpr int kMaxRowsPart = 256;
constexpr int kMaxNC = 64;
constexpr int kMaxParts = 256;
constexpr size_t kLdsBudget = 150 * 1024;

struct Plan {
    int B, Hq, Hkv, G, n, I, m, t, t_in, cap;
    int R, R_pad, NRB, m_pad, m16, PC, NC;
    int tiles_per_unit, vis_tiles, txt_tiles_per_bh, total_tiles;
    int ld_t;
    int JS, rpp, NXC, nparts, GT;
    int nvis_b, nvis_b_stride;
    float scale;
    uint16_t *S;
    float *Wp;
    float2 *stats;
    float *St;
    float *Ypart;
    size_t bytes;
};

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
            *reinterpret_cast<uint2 *>(p.S + (static_cast<size_t>(h) * p.R_pad + r) * p.m_pad + j) = make_uint2(w[0], w[1]);
        } else {
            const int tx = tile - p.vis_tiles;
            const int bh = tx / p.txt_tiles_per_bh, xt = tx - bh * p.txt_tiles_per_bh;
            const int b = bh / p.Hkv, h = bh - b * p.Hkv;
            float4 o = make_float4(acc[0] * p.scale, acc[1] * p.scale, acc[2] * p.scale, acc[3] * p.scale);
            *reinterpret_cast<float4 *>(p.St + (static_cast<size_t>(b) * p.Hq + h * p.G + g) * p.ld_t + xt * 16 + 4 * kg) = o;
        }
    }
}

// ------------------------------------------------------------------------------------------
// fb_expand: Alg. 1 steps 2 and 3 for one (KV head, 64 rows, PC positions) tile.
// ------------------------------------------------------------------------------------------
template <int PC>
__global__ __launch_bounds__(256) void fb_expand(Plan p, const uint16_t *__restrict__ theta,
                                                 const uint16_t *__restrict__ U)
{
    extern __shared__ __align__(16) uint16_t lds[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, kg = lane >> 4;

    // rb is the slow index and its stride is a multiple of 8, so the workgroups that share a
    // (head, chunk) slice of theta and U land on the same XCD and share its L2
    const int rb = blockIdx.x / p.nvis_b_stride;
    const int hc = blockIdx.x - rb * p.nvis_b_stride;
    if (hc >= p.Hkv * p.NC) return;
    const int h = hc / p.NC, pc = hc - h * p.NC;

    const int LDT = p.m_pad + 8, LDU = PC + 8;
    uint16_t *ThT = lds;                 // [PC][LDT]   theta chunk, transposed: ThT[pos][j]
    uint16_t *Ul = lds + PC * LDT;       // [m16][LDU]  U chunk: Ul[j][pos]

    // scores of this wave's 16 rows: first batch of fragments in flight during the LDS fill
    const int r0 = rb * kRB + wave * 16;
    const bool wave_live = r0 < p.R;
    const int r = r0 + r16;
    const uint16_t *srow = p.S + (static_cast<size_t>(h) * p.R_pad + r) * p.m_pad + 8 * kg;
    const int KS = p.m_pad / 32;
    constexpr int SB = 8;
    uint4 sfr[SB];
#pragma unroll
    for (int k = 0; k < SB; ++k)
        sfr[k] = (wave_live && k < KS) ? *reinterpret_cast<const uint4 *>(srow + 32 * k) : make_uint4(0, 0, 0, 0);

    // ---- stage the theta chunk (transposed) and the U chunk in LDS ------------------------------
    // a thread owns a pair of consecutive rows j, j+1 and 8 positions; the pair is packed so the
    // transposed store is one 32-bit word per position
    constexpr int SEGS = PC / 8;                 // 16-byte segments per chunk row
    constexpr int SPW = SEGS / 2;                // segments covered by one wave
    const int seg = (lane / (64 / SPW)) + SPW * (wave & 1);
    const int jp = (lane % (64 / SPW)) + (64 / SPW) * (wave >> 1);
    constexpr int JPAIRS = 2 * (64 / SPW);       // row pairs per pass
    {
        const uint16_t *th = theta + static_cast<size_t>(h) * p.m * p.n + pc * PC + 8 * seg;
        const uint16_t *uh = U + static_cast<size_t>(h) * p.m * p.n + pc * PC + 8 * seg;
        constexpr int FB = 4;                    // passes per batch: 16 loads of 16 B in flight
        for (int j0 = 2 * jp; j0 < p.m16; j0 += 2 * JPAIRS * FB) {
            uint4 tv[FB][2], uv[FB][2];
#pragma unroll
            for (int k = 0; k < FB; ++k)
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int j = j0 + 2 * JPAIRS * k + e;
                    tv[k][e] = make_uint4(0, 0, 0, 0);
                    uv[k][e] = make_uint4(0, 0, 0, 0);
                    if (j < p.m) {
                        tv[k][e] = *reinterpret_cast<const uint4 *>(th + static_cast<size_t>(j) * p.n);
                        uv[k][e] = *reinterpret_cast<const uint4 *>(uh + static_cast<size_t>(j) * p.n);
                    }
                }
#pragma unroll
            for (int k = 0; k < FB; ++k) {
                const int j = j0 + 2 * JPAIRS * k;
                if (j >= p.m16) break;
                *reinterpret_cast<uint4 *>(Ul + j * LDU + 8 * seg) = uv[k][0];
                *reinterpret_cast<uint4 *>(Ul + (j + 1) * LDU + 8 * seg) = uv[k][1];
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
        // zero the k padding of the transposed theta chunk: columns [m16, m_pad)
        const int padc = p.m_pad - p.m16;
        for (int idx = threadIdx.x; idx < PC * padc; idx += 256) {
            const int pp = idx / padc, j = p.m16 + idx - pp * padc;
            ThT[pp * LDT + j] = 0;
        }
    }
    __syncthreads();
    if (!wave_live) return;

    // ---- step 2: L^T[pos][row] = sum_j theta[j][pos] S[row][j] --------------------------------
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
            if (ks >= KS) break;
            uint4 c4 = cur[k];
            const int jb = 32 * ks + 8 * kg;
            if (jb + 8 > p.m) {     // scores beyond the compressed length do not exist
                uint32_t w[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (jb + 2 * e >= p.m) w[e] = 0;
                    else if (jb + 2 * e + 1 >= p.m) w[e] &= 0xffffu;
                }
                c4 = make_uint4(w[0], w[1], w[2], w[3]);
            }
            const bf16x8 bfrag = as_bf16x8(c4);
#pragma unroll
            for (int mt = 0; mt < PC / 16; ++mt) {
                const bf16x8 afrag = *reinterpret_cast<const bf16x8 *>(ThT + (16 * mt + r16) * LDT + 32 * ks + 8 * kg);
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, bfrag, acc[mt], 0, 0, 0);
            }
        }
    }

    // ---- tile-local softmax statistics of row r over the PC positions ---------------------------
    float mx = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < PC / 16; ++mt)
#pragma unroll
        for (int e = 0; e < 4; ++e) mx = fmaxf(mx, acc[mt][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    float sum = 0.f;
    uint4 pf[PC / 32];
#pragma unroll
    for (int kk = 0; kk < PC / 32; ++kk) {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
            // slots 0..3 come from position tile 2kk, slots 4..7 from tile 2kk+1
            const uint32_t a0 = f32_to_bf16_bits(__expf(acc[2 * kk][e] - mx));
            const uint32_t a1 = f32_to_bf16_bits(__expf(acc[2 * kk][e + 1] - mx));
            const uint32_t b0 = f32_to_bf16_bits(__expf(acc[2 * kk + 1][e] - mx));
            const uint32_t b1 = f32_to_bf16_bits(__expf(acc[2 * kk + 1][e + 1] - mx));
            sum += __uint_as_float(a0 << 16) + __uint_as_float(a1 << 16) +
                   __uint_as_float(b0 << 16) + __uint_as_float(b1 << 16);
            w[e >> 1] = a0 | (a1 << 16);
            w[2 + (e >> 1)] = b0 | (b1 << 16);
        }
        pf[kk] = make_uint4(w[0], w[1], w[2], w[3]);
    }
    sum += __shfl_xor(sum, 16, 64);
    sum += __shfl_xor(sum, 32, 64);
    const size_t tile_row = (static_cast<size_t>(h) * p.NC + pc) * p.R_pad + r;
    if (kg == 0 && r < p.R) p.stats[tile_row] = make_float2(mx, sum);

    // ---- step 3: W^T[j][row] = sum_pos U[j][pos] P[row][pos] ---------------------------------------
    float *wrow = p.Wp + tile_row * p.m_pad + 4 * kg;
    const int JT = p.m16 / 16;
    for (int jt = 0; jt < JT; ++jt) {
        f32x4 w = {0.f, 0.f, 0.f, 0.f};
        const uint16_t *ub = Ul + (16 * jt + r16) * LDU + 4 * kg;
#pragma unroll
        for (int kk = 0; kk < PC / 32; ++kk) {
            const uint2 lo = *reinterpret_cast<const uint2 *>(ub + 32 * kk);
            const uint2 hi = *reinterpret_cast<const uint2 *>(ub + 32 * kk + 16);
            const bf16x8 afrag = as_bf16x8(make_uint4(lo.x, lo.y, hi.x, hi.y));
            w = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, as_bf16x8(pf[kk]), w, 0, 0, 0);
        }
        *reinterpret_cast<float4 *>(wrow + 16 * jt) = make_float4(w[0], w[1], w[2], w[3]);
    }
}

// ------------------------------------------------------------------------------------------
// fc_output: Alg. 1 step 4 and the text part, streaming Vc / V_text once.  A workgroup owns
// a run of value rows (part of one image block, or a chunk of the text cache) and produces an
// un-normalised partial output relative to its OWN maximum, plus (max, sum): it needs no
// statistic from any other workgroup, so its loads are all independent of each other.
// Part record: [GT][D] floats of output, then [GT] maxima, then [GT] sums.
// ------------------------------------------------------------------------------------------
template <int GT>
__global__ __launch_bounds__(256) void fc_output(Plan p, const uint16_t *__restrict__ Vc,
                                                 const uint16_t *__restrict__ Vt)
{
    __shared__ float sM[GT], sS[GT];
    __shared__ float sAlpha[GT][kMaxNC];
    __shared__ float sW[GT][kMaxRowsPart];
    __shared__ float red[4][GT][D];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rg = lane >> 4, cs = lane & 15;

    const int nvis = p.B * p.Hkv * p.I * p.JS;
    int bh, i = 0, s = 0, lo, hi, part;
    const uint16_t *src;
    const bool vis = static_cast<int>(blockIdx.x) < nvis;
    if (vis) {
        const int u = blockIdx.x / p.JS;
        s = blockIdx.x - u * p.JS;
        bh = u / p.I;
        i = u - bh * p.I;
        lo = s * p.rpp;
        hi = min(p.m, lo + p.rpp);
        src = Vc + static_cast<size_t>(u) * p.m * D;
        part = i * p.JS + s;
    } else {
        const int id = blockIdx.x - nvis;
        bh = id / p.NXC;
        const int xc = id - bh * p.NXC;
        lo = xc * kXC;
        hi = min(p.t, lo + kXC);
        src = Vt + static_cast<size_t>(bh) * p.cap * D;
        part = p.I * p.JS + xc;
    }
    const int b = bh / p.Hkv, h = bh - b * p.Hkv;
    const int nrows = hi - lo;                 // >= 1 by construction of the grid
    const int niter = (nrows + 15) / 16;

    // start the HBM stream before the bookkeeping below
    constexpr int PF = 4;
    uint4 buf[PF];
    const uint4 *sp = reinterpret_cast<const uint4 *>(src) + cs;
    const int rowl = wave * 4 + rg;
#pragma unroll
    for (int k = 0; k < PF; ++k) {
        const int row = min(lo + rowl + 16 * k, hi - 1);
        buf[k] = (k < niter) ? sp[static_cast<size_t>(row) * (D / 8)] : make_uint4(0, 0, 0, 0);
    }

    if (vis) {
        // tile statistics of this block's own rows: alpha = exp(tile max - block max)
        for (int g = wave; g < p.G; g += 4) {
            const int r = (b * p.I + i) * p.G + g;
            float2 st = make_float2(-INFINITY, 0.f);
            if (lane < p.NC) st = p.stats[(static_cast<size_t>(h) * p.NC + lane) * p.R_pad + r];
            const float mx = wave_max(st.x);
            const float a = lane < p.NC ? __expf(st.x - mx) : 0.f;
            const float sm = wave_sum(st.y * a);
            if (lane < p.NC) sAlpha[g][lane] = a;
            if (lane == 0) { sM[g] = mx; sS[g] = s == 0 ? sm : 0.f; }
        }
        // partial W of the chunks, fetched while the statistics settle
        const int j = min(lo + static_cast<int>(threadIdx.x), hi - 1);
        const size_t cstride = static_cast<size_t>(p.R_pad) * p.m_pad;
        float wv[GT];
#pragma unroll
        for (int g = 0; g < GT; ++g) wv[g] = 0.f;
        for (int pc0 = 0; pc0 < p.NC; pc0 += 8) {
            float v[GT][8];
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                const int r = (b * p.I + i) * p.G + min(g, p.G - 1);
                const float *wp = p.Wp + (static_cast<size_t>(h) * p.NC * p.R_pad + r) * p.m_pad + j;
#pragma unroll
                for (int k = 0; k < 8; ++k) v[g][k] = wp[min(pc0 + k, p.NC - 1) * cstride];
            }
            if (pc0 == 0) __syncthreads();     // sAlpha ready
#pragma unroll
            for (int g = 0; g < GT; ++g)
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (pc0 + k < p.NC) wv[g] += sAlpha[min(g, p.G - 1)][pc0 + k] * v[g][k];
        }
        const bool on = lo + static_cast<int>(threadIdx.x) < hi;
#pragma unroll
        for (int g = 0; g < GT; ++g) sW[g][threadIdx.x] = (on && g < p.G) ? wv[g] : 0.f;
    } else {
        // text rows: probabilities relative to the chunk's own maximum
        const int x = lo + threadIdx.x;
        float sc[GT];
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            const size_t bg = static_cast<size_t>(b) * p.Hq + h * p.G + min(g, p.G - 1);
            sc[g] = (x < hi) ? p.St[bg * p.ld_t + x] : -INFINITY;
        }
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            const float wm = wave_max(sc[g]);
            if (lane == 0) red[wave][g][0] = wm;
        }
        __syncthreads();
        float e[GT];
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            const float mx = fmaxf(fmaxf(red[0][g][0], red[1][g][0]), fmaxf(red[2][g][0], red[3][g][0]));
            e[g] = (x < hi) ? __expf(sc[g] - mx) : 0.f;
            sW[g][threadIdx.x] = g < p.G ? e[g] : 0.f;
            const float ws = wave_sum(e[g]);
            if (lane == 0) red[wave][g][1] = ws;
            if (threadIdx.x == 0) sM[g] = mx;
        }
        __syncthreads();
        if (threadIdx.x < GT)
            sS[threadIdx.x] = red[0][threadIdx.x][1] + red[1][threadIdx.x][1] +
                              red[2][threadIdx.x][1] + red[3][threadIdx.x][1];
    }
    __syncthreads();

    // ---- stream the value rows: acc[g][c] += w[g][row] * v[row][c] ------------------------------------
    float acc[GT][8];
#pragma unroll
    for (int g = 0; g < GT; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    for (int it0 = 0; it0 < niter; it0 += PF) {
        uint4 cur[PF];
#pragma unroll
        for (int k = 0; k < PF; ++k) cur[k] = buf[k];
#pragma unroll
        for (int k = 0; k < PF; ++k) {
            const int itn = it0 + PF + k;
            const int row = min(lo + rowl + 16 * itn, hi - 1);
            if (itn < niter) buf[k] = sp[static_cast<size_t>(row) * (D / 8)];
        }
#pragma unroll
        for (int k = 0; k < PF; ++k) {
            if (it0 + k >= niter) break;
            const int jl = rowl + 16 * (it0 + k);      // < 256; weights are zero beyond the rows
            const uint32_t w4[4] = {cur[k].x, cur[k].y, cur[k].z, cur[k].w};
            float v[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) { v[2 * e] = bf_lo(w4[e]); v[2 * e + 1] = bf_hi(w4[e]); }
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                const float wg = sW[g][jl];
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[g][e] += wg * v[e];
            }
        }
    }
    __syncthreads();        // red[] was used as scratch by the text branch
#pragma unroll
    for (int g = 0; g < GT; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float a = acc[g][e];
            a += __shfl_xor(a, 16, 64);
            a += __shfl_xor(a, 32, 64);
            if (rg == 0) red[wave][g][8 * cs + e] = a;
        }
    __syncthreads();
    const int c = threadIdx.x & (D - 1), gh = threadIdx.x >> 7;
    float *yp = p.Ypart + (static_cast<size_t>(bh) * p.nparts + part) * (GT * D + 2 * GT);
    for (int g = gh; g < p.G; g += 2)
        yp[g * D + c] = red[0][g][c] + red[1][g][c] + red[2][g][c] + red[3][g][c];
    if (threadIdx.x < p.G) {
        yp[GT * D + threadIdx.x] = sM[threadIdx.x];
        yp[GT * D + GT + threadIdx.x] = sS[threadIdx.x];
    }
}

// ------------------------------------------------------------------------------------------
// fd_finalize: joint softmax over all parts of one (batch, KV head): rescale the partial
// outputs to the global maximum, normalise, add (sum P_vis) mu, store out and lse.
// ------------------------------------------------------------------------------------------
template <int GT>
__global__ __launch_bounds__(256) void fd_finalize(Plan p, const uint16_t *__restrict__ mu,
                                                   uint16_t *__restrict__ out,
                                                   float *__restrict__ lse)
{
    __shared__ float sScale[GT][kMaxParts + 4];
    __shared__ float sPv[GT], sLse[GT];
    const int bh = blockIdx.x, b = bh / p.Hkv, h = bh - b * p.Hkv;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rec = GT * D + 2 * GT;
    const float *yb = p.Ypart + static_cast<size_t>(bh) * p.nparts * rec;
    const int nvp = p.I * p.JS;
    for (int g = wave; g < p.G; g += 4) {
        float mx = -INFINITY;
        for (int pt = lane; pt < p.nparts; pt += 64) mx = fmaxf(mx, yb[static_cast<size_t>(pt) * rec + GT * D + g]);
        mx = wave_max(mx);
        float z = 0.f, zv = 0.f;
        for (int pt = lane; pt < p.nparts; pt += 64) {
            const float a = __expf(yb[static_cast<size_t>(pt) * rec + GT * D + g] - mx);
            const float sm = yb[static_cast<size_t>(pt) * rec + GT * D + GT + g] * a;
            z += sm;
            if (pt < nvp) zv += sm;
        }
        z = wave_sum(z);
        zv = wave_sum(zv);
        for (int pt = lane; pt < p.nparts; pt += 64)
            sScale[g][pt] = __expf(yb[static_cast<size_t>(pt) * rec + GT * D + g] - mx) / z;
        if (lane == 0) { sPv[g] = zv / z; sLse[g] = mx + __logf(z); }
    }
    __syncthreads();
    const int c = threadIdx.x & (D - 1), gh = threadIdx.x >> 7;
    for (int g = gh; g < p.G; g += 2) {
        float y = 0.f;
        for (int pt = 0; pt < p.nparts; ++pt) y += sScale[g][pt] * yb[static_cast<size_t>(pt) * rec + g * D + c];
        y += sPv[g] * bf_lo(mu[static_cast<size_t>(h) * D + c]);
        const size_t bg = static_cast<size_t>(b) * p.Hq + h * p.G + g;
        out[bg * D + c] = f32_to_bf16_bits(y);
        if (c == 0 && lse) lse[bg] = sLse[g];
    }
}

size_t lds_bytes(int PC, int m_pad, int m16)
{
    return (static_cast<size_t>(PC) * (m_pad + 8) + static_cast<size_t>(m16) * (PC + 8)) * sizeof(uint16_t);
}

int pick_pc(const kvc_shape &s)
{
    const int m_pad = static_cast<int>(align_up(s.m, 32)), m16 = static_cast<int>(align_up(s.m, 16));
    for (int pc : {64, 32})
        if (s.n_img_tokens % pc == 0 && s.n_img_tokens / pc <= kMaxNC && lds_bytes(pc, m_pad, m16) <= kLdsBudget)
            return pc;
    return 0;
}

Plan make_plan(const kvc_shape &s, int t, int t_in, int cap, float scale, void *base)
{
    Plan p;
    p.B = s.batch; p.Hq = s.n_q_heads; p.Hkv = s.n_kv_heads; p.G = p.Hq / p.Hkv;
    p.n = s.n_img_tokens; p.I = s.n_images; p.m = s.m;
    p.t = t; p.t_in = t_in; p.cap = cap; p.scale = scale;
    p.R = p.B * p.I * p.G;
    p.R_pad = static_cast<int>(align_up(p.R > 0 ? p.R : 1, kRB));
    p.NRB = p.I > 0 ? p.R_pad / kRB : 0;
    p.m_pad = static_cast<int>(align_up(p.m, 32));
    p.m16 = static_cast<int>(align_up(p.m, 16));
    p.PC = pick_pc(s);
    p.NC = p.PC ? p.n / p.PC : 1;
    p.tiles_per_unit = p.m16 / 16;
    p.vis_tiles = p.B * p.Hkv * p.I * p.tiles_per_unit;
    p.txt_tiles_per_bh = (t + 15) / 16;
    p.total_tiles = p.vis_tiles + p.B * p.Hkv * p.txt_tiles_per_bh;
    p.ld_t = static_cast<int>(align_up(cap > 0 ? cap : 1, 16));
    const int units = p.B * p.Hkv * p.I;
    int js = units > 0 ? (512 + units - 1) / units : 1;
    if (js > 8) js = 8;
    const int js_min = (p.m + kMaxRowsPart - 1) / kMaxRowsPart;
    if (js < js_min) js = js_min;
    p.rpp = static_cast<int>(align_up((p.m + js - 1) / js, 16));
    p.JS = (p.m + p.rpp - 1) / p.rpp;
    p.NXC = (t + kXC - 1) / kXC;
    p.nparts = p.I * p.JS + p.NXC;
    p.GT = p.G <= 1 ? 1 : p.G <= 2 ? 2 : p.G <= 4 ? 4 : p.G <= 8 ? 8 : 16;
    p.nvis_b_stride = static_cast<int>(align_up(p.Hkv * p.NC, 8));
    p.nvis_b = p.NRB * p.nvis_b_stride;

    const int nxc_max = (cap + kXC - 1) / kXC;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off += align_up(bytes, 256);
        return static_cast<char *>(base) + o;
    };
    p.S = reinterpret_cast<uint16_t *>(take(static_cast<size_t>(p.Hkv) * p.R_pad * p.m_pad * 2));
    p.Wp = reinterpret_cast<float *>(take(static_cast<size_t>(p.Hkv) * p.NC * p.R_pad * p.m_pad * 4));
    p.stats = reinterpret_cast<float2 *>(take(static_cast<size_t>(p.Hkv) * p.NC * p.R_pad * 8));
    p.St = reinterpret_cast<float *>(take(static_cast<size_t>(p.B) * p.Hq * p.ld_t * 4));
    p.Ypart = reinterpret_cast<float *>(take(static_cast<size_t>(p.B) * p.Hkv * (p.I * p.JS + nxc_max) *
                                             (p.GT * D + 2 * p.GT) * 4));
    p.bytes = off;
    return p;
}

template <int PC> kvc_status launch_b(const Plan &p, const DecodeCall &c)
{
    const size_t lds = lds_bytes(PC, p.m_pad, p.m16);
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(fb_expand<PC>),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                static_cast<int>(kLdsBudget)) != hipSuccess)
            return KVC_ERR_HIP;
        attr_set = true;
    }
    fb_expand<PC><<<p.nvis_b, 256, lds, c.stream>>>(
        p, static_cast<const uint16_t *>(c.theta), static_cast<const uint16_t *>(c.U));
    return KVC_OK;
}

template <int GT> void launch_cd(const Plan &p, const DecodeCall &c)
{
    const int grid = p.B * p.Hkv * (p.I * p.JS + p.NXC);
    fc_output<GT><<<grid, 256, 0, c.stream>>>(p, static_cast<const uint16_t *>(c.Vc),
                                             static_cast<const uint16_t *>(c.Vt));
    fd_finalize<GT><<<p.B * p.Hkv, 256, 0, c.stream>>>(p, static_cast<const uint16_t *>(c.mu),
                                                      static_cast<uint16_t *>(c.out), c.lse);
}

}  // namespace

bool fast_decode_supported(const kvc_shape &s)
{
    if (s.dtype != KVC_BF16 || s.head_dim != D) return false;
    if (s.n_q_heads / s.n_kv_heads > 16) return false;
    return pick_pc(s) != 0;
}

size_t fast_decode_ws_bytes(const kvc_shape &s, int32_t max_text)
{
    return make_plan(s, max_text, max_text, max_text, 1.f, nullptr).bytes;
}

kvc_status fast_decode(const DecodeCall &c)
{
    Plan p = make_plan(c.s, c.t, c.t_in, c.cap, c.scale, c.ws);
    if (p.nparts > kMaxParts) return generic_decode(c);   // fd_finalize keeps one scale per part in LDS
    if (p.bytes > c.ws_bytes) return KVC_ERR_WORKSPACE;
    const int waves = (p.total_tiles + kTPW - 1) / kTPW;
    fa_scores<<<(waves + 3) / 4, 256, 0, c.stream>>>(
        p, static_cast<const uint16_t *>(c.q), static_cast<const uint16_t *>(c.Kc),
        static_cast<uint16_t *>(c.Kt), static_cast<uint16_t *>(c.Vt),
        static_cast<const uint16_t *>(c.k_new), static_cast<const uint16_t *>(c.v_new));
    if (p.nvis_b > 0) {
        kvc_status st = p.PC == 64 ? launch_b<64>(p, c) : launch_b<32>(p, c);
        if (st != KVC_OK) return st;
    }
    switch (p.GT) {
    case 1: launch_cd<1>(p, c); break;
    case 2: launch_cd<2>(p, c); break;
    case 4: launch_cd<4>(p, c); break;
    case 8: launch_cd<8>(p, c); break;
    default: launch_cd<16>(p, c); break;
    }
    return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_HIP;
}

}  // namespace kvc
