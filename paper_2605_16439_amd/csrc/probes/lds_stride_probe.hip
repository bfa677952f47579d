// Standalone measurement aid (not part of libkvcapsule): cycles per LDS instruction for the access
// patterns of the matrix-core kernels (16-byte MFMA operand reads of 16 rows, row stores, the
// transposing 32-bit stores) at several row strides, 8 wavefronts per workgroup.
// Build: hipcc --offload-arch=gfx950 -O3 lds_stride_probe.hip -o lds_stride_probe   (or build.py's build_probes())
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)

// KIND 0: ds_read_b128 at byte address a; 1: ds_write_b128; 2: ds_write_b32; 3: ds_read_b64
template <int KIND> __device__ inline void access(unsigned a, u32x4 &v)
{
    if (KIND == 0) asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(a) : "memory");
    if (KIND == 1) asm volatile("ds_write_b128 %0, %1" :: "v"(a), "v"(v) : "memory");
    if (KIND == 2) asm volatile("ds_write_b32 %0, %1" :: "v"(a), "v"(v.x) : "memory");
    if (KIND == 3) { unsigned long long t; asm volatile("ds_read_b64 %0, %1" : "=v"(t) : "v"(a) : "memory"); v.x ^= (unsigned)t; }
}

// PAT: how a lane's address is formed.  S = row stride in bytes.
//  0: fragment read  : row = lane & 15, + 16 * (lane >> 4)                      (MFMA operand: 16 rows x 64 B)
//  1: row store      : row = tid >> 3,  + 16 * (tid & 7)                        (8 lanes per 128-byte row piece)
//  2: transposed b32 : word = c * (S/4) + 4 * (((w) ^ (cs >> 1)) & 7) + l4, c = 8 cs + 2 e  (the V tile's stores)
//  4: fragment read, the same 16 rows for every wavefront: row = lane & 15, + 16 * (lane >> 4)   (long rows)
//  3: fragment read, rows permuted: row = (lane & 15), + 16 * ((lane >> 4) ^ ((lane >> 1) & 3))  (XOR swizzle, unpadded rows)
template <int KIND, int PAT, int S>
__global__ __launch_bounds__(512) void k(unsigned *out, int iters)
{
    extern __shared__ __align__(16) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    unsigned a;
    if (PAT == 0) a = (16 * (wave & 3) + (lane & 15)) * S + 16 * (lane >> 4);
    else if (PAT == 1) a = (tid >> 3) * S + 16 * (tid & 7);
    else if (PAT == 2) { const int cs = lane & 15, l4 = lane >> 4; a = 4 * ((8 * cs) * (S / 4) + 4 * ((wave ^ (cs >> 1)) & 7) + l4); }
    else if (PAT == 4) a = (lane & 15) * S + 16 * (lane >> 4) + 64 * (wave & 3);
    else a = (16 * (wave & 3) + (lane & 15)) * S + 16 * ((lane >> 4) ^ ((lane >> 1) & 3));
    u32x4 v = {1u, 2u, 3u, (unsigned)tid};
    const long long t0 = clock64();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u) access<KIND>(a, v);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    const long long t1 = clock64();
    if (tid == 0 && blockIdx.x == 0) { out[0] = (unsigned)(t1 - t0); }
    if (v.x == 0x7fffffffu) out[1] = v.y;
}

template <int KIND, int PAT, int S> void run(const char *name, unsigned *out, int nt)
{
    const int iters = 2000;
    k<KIND, PAT, S><<<256, nt, 64 * 1024>>>(out, iters);
    CK(hipDeviceSynchronize());
    unsigned h[2]; CK(hipMemcpy(h, out, 8, hipMemcpyDeviceToHost));
    printf("%-34s stride %4d B, %d threads: %.1f cycles per instruction per wave (%.1f per CU-instruction)\n", name, S, nt, h[0] / (iters * 8.0), h[0] / (iters * 8.0) / (nt / 64));
    fflush(stdout);
}

int main()
{
    unsigned *out; CK(hipMalloc(&out, 256));
#define RUN(KIND, PAT, S, NAME, NT) run<KIND, PAT, S>(NAME, out, NT)
    RUN(0, 0, 144, "read_b128 fragment", 64);
    RUN(0, 0, 144, "read_b128 fragment", 512);
    RUN(0, 0, 160, "read_b128 fragment", 512);
    RUN(0, 0, 176, "read_b128 fragment", 512);
    RUN(0, 0, 192, "read_b128 fragment", 512);
    RUN(0, 0, 208, "read_b128 fragment", 512);
    RUN(0, 0, 272, "read_b128 fragment", 512);
    RUN(0, 4, 96, "read_b128 fragment, 16 rows", 512);
    RUN(0, 4, 160, "read_b128 fragment, 16 rows", 512);
    RUN(0, 4, 224, "read_b128 fragment, 16 rows", 512);
    RUN(0, 4, 288, "read_b128 fragment, 16 rows", 512);
    RUN(0, 4, 416, "read_b128 fragment, 16 rows", 512);
    RUN(0, 4, 848, "read_b128 fragment, 16 rows", 512);
    RUN(0, 4, 864, "read_b128 fragment, 16 rows", 512);
    RUN(0, 4, 880, "read_b128 fragment, 16 rows", 512);
    RUN(0, 4, 2064, "read_b128 fragment, 16 rows", 512);
    RUN(0, 4, 2080, "read_b128 fragment, 16 rows", 512);
    RUN(0, 4, 2096, "read_b128 fragment, 16 rows", 512);
    RUN(0, 4, 2112, "read_b128 fragment, 16 rows", 512);
    RUN(0, 0, 128, "read_b128 fragment (unpadded)", 512);
    RUN(0, 3, 128, "read_b128 fragment xor-swizzled", 512);
    RUN(0, 0, 64, "read_b128 contiguous rows of 64 B", 512);
    RUN(3, 0, 144, "read_b64 fragment", 512);
    RUN(1, 1, 144, "write_b128 row store", 512);
    RUN(1, 1, 160, "write_b128 row store", 512);
    RUN(1, 1, 128, "write_b128 row store (unpadded)", 512);
    RUN(2, 2, 144, "write_b32 transposed", 512);
    RUN(2, 2, 160, "write_b32 transposed", 512);
    printf("done\n");
    return 0;
}
