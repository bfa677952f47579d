// Matrix-core compress path of KVCapsule for gfx950: bf16 storage, head_dim 128.
//
// Values (Sec. 3.1, "Sequence-Level Low-Rank Compression for Values"):
//     Vc[b,h,i] = U[h] (V[b,h,block i] - 1 mu[h]^T) = U[h] V - (U[h] 1) mu[h]^T
// is one GEMM per image block, [m x n] . [n x d].  A workgroup of NW wavefronts owns up to
// 16 NW MT rows j of one block: each wavefront keeps MT tiles of 16 rows x 128 channels of
// accumulators.  Per 64 positions, the workgroup's rows of U are read with whole 128-byte
// lines and staged in LDS in row order (an MFMA operand is then 16 bytes of one row), and the
// V tile is transposed on its way into LDS (V is stored position-major, the B operand needs 8
// consecutive positions of one channel per lane).  Every LDS fragment of V feeds MT MFMAs.
// The row sums U 1 come out of the same pass as one extra MFMA against a tile of ones, already
// in the accumulator layout, so the centring costs no extra read of V.  The result is rounded
// once to bf16 and stored in the blocked channel-major layout that the decode kernel reads as
// MFMA operands.
//
// With NW = 8 two wavefronts share a SIMD: while one waits for LDS or at the barrier the other
// issues MFMAs, which a workgroup of four wavefronts (one per SIMD) cannot do.  At the shapes of
// the paper's workloads the kernel is bound by what the L2s deliver to the compute units (every
// workgroup streams its rows of U and its block of V once), not by the matrix cores.
//
// Keys (Sec. 3.1, "Selective Retention and Reconstruction for Keys"): every workgroup copies the
// key rows that the mask selects for its own rows j, 16 bytes per lane, one pass of rows per step
// of the projection, so the copy (and its writes) overlap the projection instead of preceding it.
#include "kvc_internal.h"

namespace kvc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;
constexpr int kKT = 64;        // positions per LDS tile
// Padded row of the LDS tiles in bf16 elements.  Rows 160 bytes apart are the stride at which the
// 16-byte operand reads of 16 rows meet no bank conflict (measured: 3.5 cycles per wave instruction
// against 6.0 at 144 bytes); workgroups of at most 128 rows keep 144 bytes, with which two of them fit
// one compute unit's LDS.
constexpr int ld_of(int rows) { return rows <= 128 ? kKT + 8 : kKT + 16; }
constexpr int kMaxRows = 256;  // rows of U per workgroup, at most (LDS: two stages of U and V tiles)

struct CPlan {
    int B, Hkv, n, I, m, vis0;
    int tiles, TPW, JT;         // 16-row tiles of U, tiles per workgroup, workgroups per image block
    int nproj;
    int per_xcd;                // workgroups per XCD when they divide evenly over the 8 XCDs, else 0
    int64_t sb, sh, ss;
#if defined(KVC_TIMELINE)
    unsigned long long *tl;     // timeline slots, see TSC()
#endif
};

// Developer aid, compiled in only with -DKVC_TIMELINE: thread 0 of every workgroup records the wall
// clock at a few points, in the last MiB of the workspace.
#if defined(KVC_TIMELINE)
#define TSC(K) do { if (p.tl && threadIdx.x == 0 && blockIdx.x < 1024) p.tl[blockIdx.x * 8 + (K)] = wall_clock64(); } while (0)
#else
#define TSC(K) do { } while (0)
#endif

int g_force_nw = 0, g_force_jt = 0;     // developer switches (0: the cost model decides)

__device__ inline bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// element (channel c, position p of the tile) of the transposed tile; 16-byte chunks of a row
// are XOR-swizzled with the index of the channel's 16-row MFMA tile: the transposing stores
// spread over the banks and the operand reads of one tile stay conflict-free
template <int LD> __device__ inline int sv_index(int c, int p) { return c * LD + ((((p >> 3) ^ (c >> 4)) & 7) << 3) + (p & 7); }


// NW wavefronts, MT tiles per wavefront: a workgroup covers up to 16 NW MT rows of U, so V is read
// ceil(m / (16 NW MT)) times per image block and every LDS fragment of V feeds MT MFMAs.
template <int NW, int MT>
__global__ __launch_bounds__(64 * NW) void fk_compress(CPlan p, const uint16_t *__restrict__ K,
                                                       const uint16_t *__restrict__ V,
                                                       const int32_t *__restrict__ idx,
                                                       const uint16_t *__restrict__ U,
                                                       const uint16_t *__restrict__ mu,
                                                       uint16_t *__restrict__ Kc,
                                                       uint16_t *__restrict__ Vc)
{
    constexpr int NT = 64 * NW;          // threads
    constexpr int RP = NT / 16;          // rows (or pairs of positions) one pass of 16 lanes each covers
    constexpr int NV = 512 / NT;         // V tile items (pair of positions, 8 channels) per thread
    constexpr int R = 16 * NW * MT;      // rows of U held by the workgroup
    constexpr int kLD = ld_of(R);
    extern __shared__ __align__(16) uint16_t dyn[];
    uint16_t *const sVt = dyn;                              // [2][D][kLD] V tiles, transposed
    uint16_t *const sU = dyn + 2 * D * kLD;                 // [2][R][kLD] rows of U, 64 positions each
    __shared__ int sIdx[kMaxRows];                          // mask entries of the workgroup's rows
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, kg = lane >> 4;

    // Workgroups are dealt to the 8 XCDs round-robin by the hardware.  Logical workgroups are numbered
    // so that one XCD gets a contiguous run: the JT workgroups of one image block (same V) and the
    // image blocks of one head (same U) then share an L2.
    const int bx = blockIdx.x;
    const int wg = p.per_xcd ? (bx & 7) * p.per_xcd + (bx >> 3) : bx;
    // (logical order: head, batch element, image block, so an XCD's run stays within as few heads as possible)
    const int lu = wg / p.JT, jt = wg - lu * p.JT;
    const int hb = lu / p.I, i = lu - hb * p.I;
    const int h = hb / p.B, b = hb - h * p.B;
    const int u = (b * p.Hkv + h) * p.I + i;             // the image block's index in the capsule
    const int tile0 = jt * p.TPW, ntile = min(p.TPW, p.tiles - tile0);
    // tile q of this wave is tile0 + wave + NW q; rows beyond the workgroup's share repeat the last
    // row of U and their results are dropped, so the main loop carries no tests
    int j0[MT];
#pragma unroll
    for (int q = 0; q < MT; ++q) j0[q] = 16 * (tile0 + wave + NW * q);
    // U loads: item = (row of the workgroup, 16-byte piece of its 64 positions); 2 MT per thread
    const uint16_t *usrc[2 * MT];
#pragma unroll
    for (int k = 0; k < 2 * MT; ++k) {
        const int row = (static_cast<int>(threadIdx.x) + NT * k) >> 3;
        usrc[k] = U + (static_cast<size_t>(h) * p.m + min(16 * tile0 + row, p.m - 1)) * p.n + 8 * (threadIdx.x & 7);
    }
    const int64_t blk = b * p.sb + h * p.sh + (static_cast<int64_t>(p.vis0) + static_cast<int64_t>(i) * p.n) * p.ss;
    const uint16_t *vsrc = V + blk;
    // V tile loads: item = (pair of positions, 8 channels); 512 items
    const int pair0 = threadIdx.x >> 4, cs = threadIdx.x & 15;      // further items: pair0 + RP q

    f32x4 acc[MT][8], accs[MT];
#pragma unroll
    for (int q = 0; q < MT; ++q) {
        accs[q] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) acc[q][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const uint32_t one2 = 0x3f803f80u;
    const bf16x8 ones = as_bf16x8(make_uint4(one2, one2, one2, one2));

    // Software pipeline, one barrier per step.  Step s multiplies tile s out of LDS buffer s & 1 and,
    // between its MFMAs, packs tile s + 1 from registers into the other buffer and asks memory for
    // tile s + 3 in the registers this frees: memory requests, packing and LDS stores ride under the
    // matrix work of the same wave instead of preceding it.  Two register stages rotate by name (the
    // loop is unrolled by two); X holds even tiles, Y odd ones.
    u32x4 vaX[NV][2], uaX[2 * MT], vaY[NV][2], uaY[2 * MT];
    const int NK = p.n / kKT;
    auto load_tile = [&](int kt, u32x4 (&va)[NV][2], u32x4 (&ua)[2 * MT]) {
#pragma unroll
        for (int q = 0; q < NV; ++q)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int pp = kt * kKT + 2 * (pair0 + RP * q) + e;
                va[q][e] = *(reinterpret_cast<const u32x4 *>(vsrc + static_cast<int64_t>(pp) * p.ss) + cs);
            }
#pragma unroll
        for (int k = 0; k < 2 * MT; ++k) ua[k] = *reinterpret_cast<const u32x4 *>(usrc[k] + kt * kKT);
    };
    auto store_tile = [&](int kt, const u32x4 (&va)[NV][2], const u32x4 (&ua)[2 * MT]) {
        uint16_t *buf = sVt + (kt & 1) * (D * kLD);
        uint16_t *ubuf = sU + (kt & 1) * (R * kLD);
        // transposed store: positions (2 pair, 2 pair + 1) of channel c share one 32-bit word
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            const int pl = 2 * (pair0 + RP * q);
            const uint32_t a[4] = {va[q][0].x, va[q][0].y, va[q][0].z, va[q][0].w};
            const uint32_t c2[4] = {va[q][1].x, va[q][1].y, va[q][1].z, va[q][1].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                *reinterpret_cast<uint32_t *>(buf + sv_index<kLD>(8 * cs + 2 * e, pl)) = (a[e] & 0xffffu) | (c2[e] << 16);
                *reinterpret_cast<uint32_t *>(buf + sv_index<kLD>(8 * cs + 2 * e + 1, pl)) = (a[e] >> 16) | (c2[e] & 0xffff0000u);
            }
        }
#pragma unroll
        for (int k = 0; k < 2 * MT; ++k) {
            const int row = (static_cast<int>(threadIdx.x) + NT * k) >> 3;
            *reinterpret_cast<u32x4 *>(ubuf + row * kLD + 8 * (threadIdx.x & 7)) = ua[k];
        }
    };
    // The same work in pieces, for spreading it over the MFMA groups of a step: 4 + 2 MT store pieces
    // (piece e < 4: channels 8 cs + 2 e, 8 cs + 2 e + 1 of the V items; piece 4 + k: row item k of U) and
    // 2 NV + 2 MT load items.
    constexpr int NP = 4 + 2 * MT, NL = 2 * NV + 2 * MT;
    auto store_piece = [&](int kt, const u32x4 (&va)[NV][2], const u32x4 (&ua)[2 * MT], int i) {
        uint16_t *buf = sVt + (kt & 1) * (D * kLD);
        uint16_t *ubuf = sU + (kt & 1) * (R * kLD);
        if (i < 4) {
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                const int pl = 2 * (pair0 + RP * q);
                const uint32_t a = va[q][0][i], c2 = va[q][1][i];
                *reinterpret_cast<uint32_t *>(buf + sv_index<kLD>(8 * cs + 2 * i, pl)) = (a & 0xffffu) | (c2 << 16);
                *reinterpret_cast<uint32_t *>(buf + sv_index<kLD>(8 * cs + 2 * i + 1, pl)) = (a >> 16) | (c2 & 0xffff0000u);
            }
        } else {
            const int k = i - 4;
            const int row = (static_cast<int>(threadIdx.x) + NT * k) >> 3;
            *reinterpret_cast<u32x4 *>(ubuf + row * kLD + 8 * (threadIdx.x & 7)) = ua[k];
        }
    };
    auto load_item = [&](int kt, u32x4 (&va)[NV][2], u32x4 (&ua)[2 * MT], int i) {
        if (i < 2 * NV) {
            const int q = i >> 1, e = i & 1;
            const int pp = kt * kKT + 2 * (pair0 + RP * q) + e;
            va[q][e] = *(reinterpret_cast<const u32x4 *>(vsrc + static_cast<int64_t>(pp) * p.ss) + cs);
        } else {
            const int k = i - 2 * NV;
            ua[k] = *reinterpret_cast<const u32x4 *>(usrc[k] + kt * kKT);
        }
    };
    TSC(0);
    load_tile(0, vaX, uaX);
    load_tile(min(1, NK - 1), vaY, uaY);

    // ---- keys (Sec. 3.1): Kc[u][j][:] = K[b,h, vis0 + i n + M[j], :] for this workgroup's rows j -------
    // 16 lanes per row, RP rows per pass, 4 MT passes, one pass per step of the projection: tick t
    // stores the rows of pass t, requested one step earlier, and requests those of pass t + 1.  The mask
    // entries sit in LDS (a load that depends on a load would wait in the middle of a step).  Nothing
    // here is conditional: a pass or a row beyond the workgroup's last repeats the last one (same
    // source, same destination, same bytes), because a memory operation under a run-time test makes
    // the compiler wait for every load in flight at the end of the test, the tile prefetch included.
    constexpr int P = 4 * MT;
    const int rl = threadIdx.x >> 4;
    const int jlast = min(16 * (tile0 + ntile), p.m) - 1;
    for (int r = threadIdx.x; r < R; r += NT)
        sIdx[r] = min(max(idx[min(16 * tile0 + r, jlast)], 0), p.n - 1);      // an index outside the block must not leave it
    u32x4 kvrow = *(reinterpret_cast<const u32x4 *>(K + blk + static_cast<int64_t>(min(max(idx[min(16 * tile0 + rl, jlast)], 0), p.n - 1)) * p.ss) + cs);
    auto keys_tick = [&](int t) {
        const int ps = min(t, P - 1), pl = min(t + 1, P - 1);
        const int j = min(16 * tile0 + RP * ps + rl, jlast);
        *(reinterpret_cast<u32x4 *>(Kc + (static_cast<size_t>(u) * p.m + j) * D) + cs) = kvrow;
        kvrow = *(reinterpret_cast<const u32x4 *>(K + blk + static_cast<int64_t>(sIdx[RP * pl + rl]) * p.ss) + cs);
    };

    // One step = 16 groups of MFMAs (group f: fragment f = 8 ks + nt of V against the MT tiles of U).
    // On entry the first fragments of tile kt (U for ks = 0, V fragments 0 .. AH-1) are in registers and
    // tile kt is complete in LDS buffer kt & 1.  Between the groups: the remaining fragments, AH ahead of
    // their use; tile kt + 1 packed into the other buffer piece by piece; the key rows; the barrier after
    // group kBar (all of tile kt + 1 stored, all of tile kt read); then the first fragments of tile
    // kt + 1 and the requests for tile kt + 3.  The order is pinned with scheduling barriers: left alone,
    // the compiler waits for every fragment right after asking for it.
#ifndef EXP_AH
#define EXP_AH 4
#endif
    constexpr int AH = EXP_AH, kBar = 11, PRE = 16 - kBar - 1;   // fragments of V in flight ahead; barrier group; fragments preloaded before a step
    constexpr int F0 = NP <= 10 ? 1 : 0;                 // group of the first store piece
    constexpr int FL = NP <= 9 ? 10 : 12;                // group of the first tile request
    constexpr int LPG = (NL + (16 - FL) - 1) / (16 - FL);
    constexpr int FK = NP <= 8 ? 9 : 13;                 // group of the key rows
    static_assert(F0 + NP <= kBar + 1 && FL + (NL + LPG - 1) / LPG <= 16, "pieces fit their groups");
    bf16x8 af[2][MT], bq[16];
    auto frag_u = [&](int kt, int ks, int q) {
        const uint16_t *ubuf = sU + (kt & 1) * (R * kLD);
        return *reinterpret_cast<const bf16x8 *>(ubuf + (16 * (wave + NW * q) + r16) * kLD + 32 * ks + 8 * kg);
    };
    auto frag_v = [&](int kt, int f) {       // fragment f = 8 ks + nt
        const uint16_t *buf = sVt + (kt & 1) * (D * kLD);
        return *reinterpret_cast<const bf16x8 *>(buf + sv_index<kLD>(16 * (f & 7) + r16, 32 * (f >> 3) + 8 * kg));
    };
    auto first_fragments = [&](int kt) {
#pragma unroll
        for (int q = 0; q < MT; ++q) af[0][q] = frag_u(kt, 0, q);
    };
    auto step = [&](int kt, u32x4 (&va)[NV][2], u32x4 (&ua)[2 * MT]) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int f = 0; f < 16; ++f) {
            if (f == 0) {
#pragma unroll
                for (int q = 0; q < MT; ++q) af[1][q] = frag_u(kt, 1, q);
            }
            if (f == 0) {
#pragma unroll
                for (int g = PRE; g < AH; ++g) bq[g] = frag_v(kt, g);
            }
            if (f + AH < 16) bq[f + AH] = frag_v(kt, f + AH);
            if (f == kBar + 1) first_fragments(kt + 1);
            if (f > kBar) bq[f - kBar - 1] = frag_v(kt + 1, f - kBar - 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < MT; ++q)
                acc[q][f & 7] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[f >> 3][q], bq[f], acc[q][f & 7], 0, 0, 0);
            if ((f & 7) == 7) {
#pragma unroll
                for (int q = 0; q < MT; ++q)
                    accs[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[f >> 3][q], ones, accs[q], 0, 0, 0);
            }
            // past the end: the last tile again, stored where nobody reads it
            if (f >= F0 && f < F0 + NP) store_piece(kt + 1, va, ua, f - F0);
            if (f == FK) keys_tick(kt);
            if (f >= FL) {
#pragma unroll
                for (int i = (f - FL) * LPG; i < (f - FL + 1) * LPG; ++i)
                    if (i < NL) load_item(min(kt + 3, NK - 1), va, ua, i);
            }
            // only LDS is handed over: wait for this wave's LDS traffic, then for the other waves
            // (__syncthreads() would also wait for the global loads in flight)
            if (f == kBar) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    store_tile(0, vaX, uaX);
    load_tile(min(2, NK - 1), vaX, uaX);
    uint16_t mur[8];                                     // the channel means the epilogue needs, requested early
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) mur[nt] = mu[static_cast<size_t>(h) * D + 16 * nt + r16];
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    first_fragments(0);
#pragma unroll
    for (int f = 0; f < PRE; ++f) bq[f] = frag_v(0, f);
    TSC(1);
    int kt = 0;
    for (; kt + 2 <= NK; kt += 2) {                      // no tests inside the loop body
        step(kt, vaY, uaY);
        step(kt + 1, vaX, uaX);
    }
    if (kt < NK) {
        step(kt, vaY, uaY);
        ++kt;
    }
    TSC(4);
    for (; kt < P; ++kt) keys_tick(kt);                  // passes a short block left over

    // ---- epilogue: centre, round once, store in the blocked layout -----------------------------------
    // lane holds rows j = j0 + 4 kg + e (e = 0..3) of channel c = 16 nt + r16; accs[e] = sum_p U[j][p]
    float muc[8];
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) muc[nt] = __uint_as_float(static_cast<uint32_t>(mur[nt]) << 16);
#pragma unroll
    for (int q = 0; q < MT; ++q) {
        if (wave + NW * q >= ntile) continue;
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
    TSC(5);
}

template <int NW, int MT> bool launch(const CPlan &p, const CompressCall &c)
{
    static_assert(16 * NW * MT <= kMaxRows, "rows of U per workgroup");
    const size_t lds = static_cast<size_t>(2) * (D + 16 * NW * MT) * ld_of(16 * NW * MT) * sizeof(uint16_t);
    static bool attr_set[kMaxDevices] = {};
    if (!allow_lds(reinterpret_cast<const void *>(fk_compress<NW, MT>), lds, attr_set)) return false;
    fk_compress<NW, MT><<<p.nproj, 64 * NW, lds, c.stream>>>(
        p, static_cast<const uint16_t *>(c.K), static_cast<const uint16_t *>(c.V), c.key_idx,
        static_cast<const uint16_t *>(c.U), static_cast<const uint16_t *>(c.mu),
        static_cast<uint16_t *>(c.Kc), static_cast<uint16_t *>(c.Vc));
    return true;
}

// compute units of the current device, asked once per device
int device_cus()
{
    static int cus[kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
    if (cus[dev] == 0) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) {
            (void)hipGetLastError();
            v = 256;
        }
        cus[dev] = v;
    }
    return cus[dev];
}

}  // namespace

void fast_compress_knobs(int nw, int jt)
{
    if (nw >= 0) g_force_nw = nw;
    if (jt >= 0) g_force_jt = jt;
}

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
    // The 16-row tiles of U are shared out evenly over JT workgroups per image block, at most 16 per
    // workgroup.  A workgroup's time has a part that does not depend on its share (it streams the
    // whole block of V) and a part that grows with it, about 20 : 1 per tile on MI355X; JT minimises
    // rounds of resident workgroups (one per compute unit) times that cost, which at the paper's shapes
    // is the smallest JT the kernel supports.
    p.tiles = (s.m + 15) / 16;
    const int units = p.B * p.Hkv * p.I;
    const int max_tpw = kMaxRows / 16;
    {
        const int cus = device_cus();
        const int jt_min = (p.tiles + max_tpw - 1) / max_tpw, jt_max = (p.tiles + 3) / 4;
        long best = -1;
        for (int jt = jt_min; jt <= jt_max; ++jt) {
            const int tpw = (p.tiles + jt - 1) / jt;
            const long rounds = (static_cast<long>(units) * jt + cus - 1) / cus;
            const long cost = rounds * (20 + tpw);
            if (best < 0 || cost < best) { best = cost; p.JT = jt; }
        }
        if (g_force_jt > 0) p.JT = std::min(std::max(g_force_jt, jt_min), p.tiles);
    }
    p.TPW = (p.tiles + p.JT - 1) / p.JT;
    p.nproj = units * p.JT;
    p.per_xcd = p.nproj % 8 == 0 ? p.nproj / 8 : 0;
    p.sb = c.stride_b; p.sh = c.stride_h; p.ss = c.stride_s;
#if defined(KVC_TIMELINE)
    p.tl = (c.ws && c.ws_bytes >= (2u << 20))
               ? reinterpret_cast<unsigned long long *>((reinterpret_cast<uintptr_t>(c.ws) + c.ws_bytes - (1u << 20)) & ~uintptr_t(7))
               : nullptr;
#endif
    const int nw = g_force_nw == 4 || g_force_nw == 8 ? g_force_nw : (p.TPW > 4 ? 8 : 4);
    bool ok;
    if (nw == 8) {
        ok = p.TPW > 8 ? launch<8, 2>(p, c) : launch<8, 1>(p, c);
    } else {
        switch ((p.TPW + 3) / 4) {
        case 1: ok = launch<4, 1>(p, c); break;
        case 2: ok = launch<4, 2>(p, c); break;
        case 3: ok = launch<4, 3>(p, c); break;
        default: ok = launch<4, 4>(p, c); break;
        }
    }
    return ok && hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_HIP;
}

}  // namespace kvc
