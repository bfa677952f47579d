// Matrix-core compress path of KVCapsule for gfx950: bf16 storage, head_dim 128.
//
// Values (Sec. 3.1, "Sequence-Level Low-Rank Compression for Values"):
//     Vc[b,h,i] = U[h] (V[b,h,block i] - 1 mu[h]^T) = U[h] V - (U[h] 1) mu[h]^T
// is one GEMM per image block, [m x n] . [n x d].  A workgroup owns up to 64 MT rows j of one
// block (MT <= 4): each of its 4 wavefronts keeps MT tiles of 16 rows x 128 channels of
// accumulators.  Per 64 positions, the workgroup's rows of U are read with whole 128-byte
// lines and staged in LDS in row order (an MFMA operand is then 16 bytes of one row), and the
// V tile is transposed on its way into LDS (V is stored position-major, the B operand needs 8
// consecutive positions of one channel per lane).  Every LDS fragment of V feeds MT MFMAs.  The row sums U 1 come out of the same pass as one extra MFMA against a tile of
// ones, already in the accumulator layout, so the centring costs no extra read of V.
// The result is rounded once to bf16 and stored in the blocked channel-major layout that the
// decode kernel reads as MFMA operands.
//
// Keys (Sec. 3.1, "Selective Retention and Reconstruction for Keys"): every workgroup first copies
// the key rows that the mask selects for its own rows j, 16 bytes per lane.
#include "kvc_internal.h"

namespace kvc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;
constexpr int kKT = 64;        // positions per LDS tile
constexpr int kLD = kKT + 8;   // padded row of the transposed V tile (bf16 elements)
constexpr int kMaxMT = 4;      // 16-row tiles of U per wavefront, at most

struct CPlan {
    int B, Hkv, n, I, m, vis0;
    int tiles, TPW, JT;         // 16-row tiles of U, tiles per workgroup, workgroups per image block
    int nproj;
    int64_t sb, sh, ss;
};

__device__ inline bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// element (channel c, position p of the tile) of the transposed tile; 16-byte chunks of a row
// are XOR-swizzled with the index of the channel's 16-row MFMA tile: the transposing stores
// spread over the banks and the operand reads of one tile stay conflict-free
__device__ inline int sv_index(int c, int p) { return c * kLD + ((((p >> 3) ^ (c >> 4)) & 7) << 3) + (p & 7); }

// MT = tiles per wavefront: a workgroup covers up to 64 MT rows of U, so V is read
// ceil(m / (64 MT)) times per image block and every LDS fragment of V feeds MT MFMAs.
template <int MT>
__global__ __launch_bounds__(256) void fk_compress(CPlan p, const uint16_t *__restrict__ K,
                                                   const uint16_t *__restrict__ V,
                                                   const int32_t *__restrict__ idx,
                                                   const uint16_t *__restrict__ U,
                                                   const uint16_t *__restrict__ mu,
                                                   uint16_t *__restrict__ Kc,
                                                   uint16_t *__restrict__ Vc)
{
    __shared__ __align__(16) uint16_t sVt[2][D * kLD];
    extern __shared__ __align__(16) uint16_t sU[];          // [2][64 MT][kLD] rows of U, 64 positions each
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, kg = lane >> 4;

    // ---------------- values: up to 4 MT tiles of 16 rows j of one image block ----------------
    const int u = blockIdx.x / p.JT, jt = blockIdx.x - u * p.JT;
    const int bh = u / p.I, i = u - bh * p.I;
    const int b = bh / p.Hkv, h = bh - b * p.Hkv;
    const int tile0 = jt * p.TPW, ntile = min(p.TPW, p.tiles - tile0);
    // tile q of this wave is tile0 + wave + 4 q; rows beyond the workgroup's share repeat the last
    // row of U and their results are dropped, so the main loop carries no tests
    int j0[MT];
#pragma unroll
    for (int q = 0; q < MT; ++q) j0[q] = 16 * (tile0 + wave + 4 * q);
    // U loads: item = (row of the workgroup, 16-byte piece of its 64 positions); 2 MT per thread
    const uint16_t *usrc[2 * MT];
#pragma unroll
    for (int k = 0; k < 2 * MT; ++k) {
        const int row = (static_cast<int>(threadIdx.x) + 256 * k) >> 3;
        usrc[k] = U + (static_cast<size_t>(h) * p.m + min(16 * tile0 + row, p.m - 1)) * p.n + 8 * (threadIdx.x & 7);
    }
    // ---- keys (Sec. 3.1): Kc[u][j][:] = K[b,h, vis0 + i n + M[j], :] for this workgroup's rows j -------
    // 16 lanes per row, 16 rows per pass; all rows are requested before the first is stored, and the
    // stores drain while the projection below starts
    {
        const uint16_t *ksrc = K + b * p.sb + h * p.sh + (static_cast<int64_t>(p.vis0) + static_cast<int64_t>(i) * p.n) * p.ss;
        const int rl = threadIdx.x >> 4, c16 = threadIdx.x & 15;
        const int jend = min(16 * (tile0 + ntile), p.m);
        u32x4 kv[4 * MT];
#pragma unroll
        for (int k = 0; k < 4 * MT; ++k) {
            const int j = min(16 * (tile0 + k) + rl, p.m - 1);
            const int row = min(max(idx[j], 0), p.n - 1);      // an index outside the block must not leave it
            kv[k] = *(reinterpret_cast<const u32x4 *>(ksrc + static_cast<int64_t>(row) * p.ss) + c16);
        }
#pragma unroll
        for (int k = 0; k < 4 * MT; ++k) {
            const int j = 16 * (tile0 + k) + rl;
            if (j < jend) *(reinterpret_cast<u32x4 *>(Kc + (static_cast<size_t>(u) * p.m + j) * D) + c16) = kv[k];
        }
    }
    const uint16_t *vsrc = V + b * p.sb + h * p.sh + (static_cast<int64_t>(p.vis0) + static_cast<int64_t>(i) * p.n) * p.ss;
    // V tile loads: item = (pair of positions, 8 channels); 512 items, two per thread
    const int pair0 = threadIdx.x >> 4, cs = threadIdx.x & 15;      // second item: pair0 + 16

    f32x4 acc[MT][8], accs[MT];
#pragma unroll
    for (int q = 0; q < MT; ++q) {
        accs[q] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) acc[q][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const uint32_t one2 = 0x3f803f80u;
    const bf16x8 ones = as_bf16x8(make_uint4(one2, one2, one2, one2));

    // Two register stages rotate by name (the loop is unrolled by two): a tile's loads are issued
    // right after the barrier of the previous tile and have that tile's MFMA work to arrive; nothing
    // is copied between stages.
    u32x4 vaA[2][2], uaA[2 * MT], vaB[2][2], uaB[2 * MT];
    auto load_tile = [&](int kt, u32x4 (&va)[2][2], u32x4 (&ua)[2 * MT]) {
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int pp = kt * kKT + 2 * (pair0 + 16 * q) + e;
                va[q][e] = *(reinterpret_cast<const u32x4 *>(vsrc + static_cast<int64_t>(pp) * p.ss) + cs);
            }
#pragma unroll
        for (int k = 0; k < 2 * MT; ++k) ua[k] = *reinterpret_cast<const u32x4 *>(usrc[k] + kt * kKT);
    };
    const int NK = p.n / kKT;
    auto step = [&](int kt, u32x4 (&va)[2][2], u32x4 (&ua)[2 * MT]) {
        uint16_t *buf = sVt[kt & 1];
        uint16_t *ubuf = sU + (kt & 1) * (64 * MT * kLD);
        // transposed store: positions (2 pair, 2 pair + 1) of channel c share one 32-bit word
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int pl = 2 * (pair0 + 16 * q);
            const uint32_t a[4] = {va[q][0].x, va[q][0].y, va[q][0].z, va[q][0].w};
            const uint32_t c2[4] = {va[q][1].x, va[q][1].y, va[q][1].z, va[q][1].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                *reinterpret_cast<uint32_t *>(buf + sv_index(8 * cs + 2 * e, pl)) = (a[e] & 0xffffu) | (c2[e] << 16);
                *reinterpret_cast<uint32_t *>(buf + sv_index(8 * cs + 2 * e + 1, pl)) = (a[e] >> 16) | (c2[e] & 0xffff0000u);
            }
        }
#pragma unroll
        for (int k = 0; k < 2 * MT; ++k) {
            const int row = (static_cast<int>(threadIdx.x) + 256 * k) >> 3;
            *reinterpret_cast<u32x4 *>(ubuf + row * kLD + 8 * (threadIdx.x & 7)) = ua[k];
        }
        __syncthreads();
        load_tile(min(kt + 2, NK - 1), va, ua);          // past the end: the last tile again, unused
        // every fragment of the tile is requested from LDS before the first MFMA: the reads of one
        // wave then overlap the matrix work instead of being waited for one by one
        bf16x8 af[2][MT], bq[2][8];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int q = 0; q < MT; ++q)
                af[ks][q] = *reinterpret_cast<const bf16x8 *>(ubuf + (16 * (wave + 4 * q) + r16) * kLD + 32 * ks + 8 * kg);
#pragma unroll
            for (int nt = 0; nt < 8; ++nt)
                bq[ks][nt] = *reinterpret_cast<const bf16x8 *>(buf + sv_index(16 * nt + r16, 32 * ks + 8 * kg));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int nt = 0; nt < 8; ++nt)
#pragma unroll
                for (int q = 0; q < MT; ++q)
                    acc[q][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[ks][q], bq[ks][nt], acc[q][nt], 0, 0, 0);
#pragma unroll
            for (int q = 0; q < MT; ++q)
                accs[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[ks][q], ones, accs[q], 0, 0, 0);
        }
    };
    load_tile(0, vaA, uaA);
    load_tile(min(1, NK - 1), vaB, uaB);
    int kt = 0;
    for (; kt + 2 <= NK; kt += 2) {                      // no tests inside the loop body
        step(kt, vaA, uaA);
        step(kt + 1, vaB, uaB);
    }
    if (kt < NK) step(kt, vaA, uaA);

    // ---- epilogue: centre, round once, store in the blocked layout -----------------------------------
    // lane holds rows j = j0 + 4 kg + e (e = 0..3) of channel c = 16 nt + r16; accs[e] = sum_p U[j][p]
    float muc[8];
#pragma unroll
    for (int nt = 0; nt < 8; ++nt)
        muc[nt] = __uint_as_float(static_cast<uint32_t>(mu[static_cast<size_t>(h) * D + 16 * nt + r16]) << 16);
#pragma unroll
    for (int q = 0; q < MT; ++q) {
        if (wave + 4 * q >= ntile) continue;
        const int jb = (j0[q] + 4 * kg) >> 3, jr = (j0[q] + 4 * kg) & 7;
        const int w = min(8, p.m - 8 * jb);                     // width of the block these rows sit in
        uint16_t *vout = Vc + static_cast<size_t>(u) * p.m * D + static_cast<size_t>(jb) * 8 * D;
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
            const int c = 16 * nt + r16;
            uint32_t o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = f32_to_bf16_bits(acc[q][nt][e] - accs[q][e] * muc[nt]);
            if (w == 8) {
                *reinterpret_cast<uint2 *>(vout + c * 8 + jr) = make_uint2(o[0] | (o[1] << 16), o[2] | (o[3] << 16));
            } else if (w > 0) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (jr + e < w) vout[c * w + jr + e] = static_cast<uint16_t>(o[e]);
            }
        }
    }
}

template <int MT> bool launch(const CPlan &p, const CompressCall &c)
{
    const size_t lds = static_cast<size_t>(2) * 64 * MT * kLD * sizeof(uint16_t);
    static bool attr_set[kMaxDevices] = {};
    if (!allow_lds(reinterpret_cast<const void *>(fk_compress<MT>), lds, attr_set)) return false;
    fk_compress<MT><<<p.nproj, 256, lds, c.stream>>>(
        p, static_cast<const uint16_t *>(c.K), static_cast<const uint16_t *>(c.V), c.key_idx,
        static_cast<const uint16_t *>(c.U), static_cast<const uint16_t *>(c.mu),
        static_cast<uint16_t *>(c.Kc), static_cast<uint16_t *>(c.Vc));
    return true;
}

}  // namespace

bool fast_compress_supported(const kvc_shape &s)
{
    return s.dtype == KVC_BF16 && s.head_dim == D && s.n_img_tokens % kKT == 0;
}

size_t fast_compress_ws_bytes(const kvc_shape &) { return 0; }

kvc_status fast_compress(const CompressCall &c)
{
    const kvc_shape &s = c.s;
    if (s.n_images == 0) return KVC_OK;
    CPlan p;
    p.B = s.batch; p.Hkv = s.n_kv_heads; p.n = s.n_img_tokens; p.I = s.n_images; p.m = s.m;
    p.vis0 = c.vis_start;
    // The 16-row tiles of U are shared out evenly over JT workgroups per image block, each wave taking
    // MT = ceil(tiles per workgroup / 4) of them.  JT is chosen by a small cost model fitted to
    // measurements on MI355X: time per round of resident workgroups grows with MT (fewer, fatter
    // workgroups read V less often but leave one workgroup per CU), MT = 1 fits two per CU.
    p.tiles = (s.m + 15) / 16;
    const int units = p.B * p.Hkv * p.I;
    {
        static const int round_cost[kMaxMT + 1] = {0, 27, 30, 36, 42};
        const int cus = 256;
        long best = -1;
        for (int jt = (p.tiles + 4 * kMaxMT - 1) / (4 * kMaxMT); jt <= (p.tiles + 3) / 4; ++jt) {
            const int tpw = (p.tiles + jt - 1) / jt, mt = (tpw + 3) / 4;
            const long slots = mt == 1 ? 2L * cus : cus;
            const long rounds = (static_cast<long>(units) * jt + slots - 1) / slots;
            const long cost = rounds * round_cost[mt];
            if (best < 0 || cost < best) { best = cost; p.JT = jt; }
        }
    }
    p.TPW = (p.tiles + p.JT - 1) / p.JT;
    p.nproj = units * p.JT;
    p.sb = c.stride_b; p.sh = c.stride_h; p.ss = c.stride_s;
    bool ok;
    switch ((p.TPW + 3) / 4) {
    case 1: ok = launch<1>(p, c); break;
    case 2: ok = launch<2>(p, c); break;
    case 3: ok = launch<3>(p, c); break;
    default: ok = launch<4>(p, c); break;
    }
    return ok && hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_HIP;
}

}  // namespace kvc
