// Standalone measurement aid (not part of libkvcapsule): the rate at which a compute unit of an MI355X
// pulls L2-resident data through its L1, for several access forms and numbers of bytes in flight.
// Every workgroup streams over its own slice (slice_kb per workgroup, reps times); slices of 64 KB
// stay in the XCD's L2 and do not fit the L1.
// Build: hipcc --offload-arch=gfx950 -O3 l2_fill_probe.hip -o l2_fill_probe   (or build.py's build_probes())
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)

// mode 0: dwordx4 loads, UN in flight per thread; mode 1: dwordx2; mode 2: LDS-DMA 16 B per lane
template <int UN, int MODE>
__global__ void probe(const unsigned char *__restrict__ src, unsigned *__restrict__ sink, int slice_bytes, int reps, int wg_stride_slices)
{
    extern __shared__ __align__(16) unsigned char lds[];
    const unsigned char *base = src + static_cast<size_t>(blockIdx.x % wg_stride_slices) * slice_bytes;
    const int nt = blockDim.x;
    unsigned acc = 0;
    constexpr int W = MODE == 1 ? 8 : 16;
    const int per_iter = nt * W * UN;                 // bytes per unrolled iteration of the workgroup
    const int iters = slice_bytes / per_iter;
    for (int r = 0; r < reps; ++r) {
        for (int it = 0; it < iters; ++it) {
            const unsigned char *p = base + static_cast<size_t>(it) * per_iter + threadIdx.x * W;
            if (MODE == 0) {
                u32x4 v[UN];
#pragma unroll
                for (int k = 0; k < UN; ++k) v[k] = *reinterpret_cast<const u32x4 *>(p + static_cast<size_t>(k) * nt * W);
#pragma unroll
                for (int k = 0; k < UN; ++k) acc += v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
            } else if (MODE == 1) {
                u32x2 v[UN];
#pragma unroll
                for (int k = 0; k < UN; ++k) v[k] = *reinterpret_cast<const u32x2 *>(p + static_cast<size_t>(k) * nt * W);
#pragma unroll
                for (int k = 0; k < UN; ++k) acc += v[k].x ^ v[k].y;
            } else {
                // each wave's instruction writes 1 KB of LDS at (wave base + k * nt * 16)
#pragma unroll
                for (int k = 0; k < UN; ++k)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p + static_cast<size_t>(k) * nt * W),
                                                     (__attribute__((address_space(3))) void *)(lds + (threadIdx.x >> 6) * 1024 + k * nt * 16), 16, 0, 0);
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                acc += lds[threadIdx.x * 4];
            }
        }
    }
    if (acc == 0x12345678u) sink[0] = acc;
}

template <int UN, int MODE> void run(const char *name, const unsigned char *src, unsigned *sink, int nwg, int nt, int slice_kb, int reps, int nslices)
{
    const int slice = slice_kb * 1024;
    const size_t lds = MODE == 2 ? static_cast<size_t>(UN) * nt * 16 : 0;
    if (lds > 64 * 1024) return;
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    probe<UN, MODE><<<nwg, nt, lds>>>(src, sink, slice, 2, nslices);
    CK(hipDeviceSynchronize());
    float best = 1e30f;
    for (int t = 0; t < 3; ++t) {
        CK(hipEventRecord(e0));
        probe<UN, MODE><<<nwg, nt, lds>>>(src, sink, slice, reps, nslices);
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1)); if (ms < best) best = ms;
    }
    constexpr int W = MODE == 1 ? 8 : 16;
    const int per_iter = nt * W * UN, iters = slice / per_iter;
    if (iters == 0) return;
    const double bytes = static_cast<double>(nwg) * iters * per_iter * reps;
    printf("%-14s wg=%4d threads=%4d unroll=%2d slice=%4d KB: %8.1f us  %7.2f TB/s  %6.1f GB/s per WG\n", name, nwg, nt, UN, slice_kb,
           best * 1e3, bytes / (best * 1e-3) / 1e12, bytes / nwg / (best * 1e-3) / 1e9);
    fflush(stdout);
}

int main()
{
    const size_t total = 256u << 20;
    unsigned char *src; unsigned *sink;
    CK(hipMalloc(&src, total)); CK(hipMalloc(&sink, 256)); CK(hipMemset(src, 1, total));
    const int reps = 64;
    // private slices, L2-resident per XCD: nwg slices of slice_kb (32 per XCD)
    for (int nwg : {32, 64, 128, 256, 512}) {
        run<4, 0>("x4", src, sink, nwg, 256, 64, reps, nwg);
        run<8, 0>("x4", src, sink, nwg, 256, 64, reps, nwg);
    }
    for (int nt : {256, 512, 1024}) {
        run<2, 0>("x4", src, sink, 256, nt, 64, reps, 256);
        run<4, 0>("x4", src, sink, 256, nt, 64, reps, 256);
        run<8, 0>("x4", src, sink, 256, nt, 64, reps, 256);
        run<16, 0>("x4", src, sink, 256, nt, 64, reps, 256);
        run<8, 1>("x2", src, sink, 256, nt, 64, reps, 256);
        run<4, 2>("lds-dma", src, sink, 256, nt, 64, reps, 256);
        run<8, 2>("lds-dma", src, sink, 256, nt, 64, reps, 256);
    }
    // shared slices: all workgroups of an XCD class read the same 8 slices (L2 hot lines shared)
    run<8, 0>("x4 shared8", src, sink, 256, 256, 64, reps, 8);
    run<8, 0>("x4 shared8", src, sink, 256, 512, 64, reps, 8);
    // slices that fit the L1 (16 KB): L1 hit rate
    run<8, 0>("x4 L1-fit", src, sink, 256, 256, 16, reps * 4, 256);
    // larger slices: 1 MB per workgroup = 256 MB total: memory-side cache / HBM
    run<8, 0>("x4 hbm", src, sink, 256, 256, 1024, 4, 256);
    run<8, 0>("x4 hbm", src, sink, 256, 512, 1024, 4, 256);
    run<8, 0>("x4 hbm", src, sink, 512, 512, 512, 4, 512);
    CK(hipDeviceSynchronize());
    printf("done\n");
    return 0;
}
