// LDS read rate (ds_read_b128, conflict-free) per compute unit with 4 and 8 reading waves, alone and
// while other waves stream direct-to-LDS loads from L2 into another part of the LDS: do the two
// share the LDS's time?  Prints bytes per shader clock per CU for both.  Stand-alone:
// hipcc --offload-arch=gfx950 -O3.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
static __device__ __forceinline__ void load_to_lds(u32x4 desc, unsigned voff, unsigned soff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" : : "s"(lds_addr), "v"(voff), "s"(desc), "s"(soff) : "memory", "m0");
}
static __device__ __forceinline__ u32x4 make_desc(const void *p, unsigned bytes) {
    const unsigned long long v = reinterpret_cast<unsigned long long>(p);
    return u32x4{(unsigned)v, (unsigned)(v >> 32) & 0xffffu, bytes, 0x00020000u};
}
extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
// waves [0, DW): DMA loaders, 8 x 1 KiB per round into the upper 64 KiB; waves [DW, DW+RW): readers,
// 8 ds_read_b128 (linear, conflict-free) per round from the lower 64 KiB.  mode bit 0: loaders run, bit 1: readers run.
template <int DW, int RW>
__global__ __launch_bounds__(64 * (DW + RW)) void k(const char* src, unsigned src_bytes, int iters, int mode, long long* ticks, unsigned* sink) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)lds;
    for (int i = threadIdx.x; i < 65536 / 16; i += 64 * (DW + RW)) reinterpret_cast<u32x4*>(lds)[i] = u32x4{(unsigned)i, 1u, 2u, 3u};
    __syncthreads();
    u32x4 acc = {0, 0, 0, 0};
    const long long t0 = clock64();
    if (wave < DW) {
        if (mode & 1) {
            const u32x4 d = make_desc(src, src_bytes);
            unsigned so = 0;
            for (int it = 0; it < iters; ++it) {
#pragma unroll
                for (int j = 0; j < 8; ++j) load_to_lds(d, blockIdx.x * 65536u + (wave * 8 + j) * 1024u + lane * 16u, so, lds_base + 65536u + ((wave * 8 + j) & 63) * 1024u);
                asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
                so += DW * 8192u; if (so + DW * 8192u > 65536u) so = 0;
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
    } else if (mode & 2) {
        unsigned off[8];
        for (int j = 0; j < 8; ++j) off[j] = lds_base + (((wave - DW) * 8 + j) & 63) * 1024u + lane * 16u;
        u32x4 v[8];
        for (int it = 0; it < iters; ++it) {
            asm volatile("ds_read_b128 %0, %8\n ds_read_b128 %1, %9\n ds_read_b128 %2, %10\n ds_read_b128 %3, %11\n ds_read_b128 %4, %12\n ds_read_b128 %5, %13\n ds_read_b128 %6, %14\n ds_read_b128 %7, %15\n s_waitcnt lgkmcnt(0)"
                         : "=v"(v[0]), "=v"(v[1]), "=v"(v[2]), "=v"(v[3]), "=v"(v[4]), "=v"(v[5]), "=v"(v[6]), "=v"(v[7])
                         : "v"(off[0]), "v"(off[1]), "v"(off[2]), "v"(off[3]), "v"(off[4]), "v"(off[5]), "v"(off[6]), "v"(off[7]) : "memory");
            for (int j = 0; j < 8; ++j) acc ^= v[j];
        }
    }
    const long long t1 = clock64();
    if (lane == 0) { ticks[(blockIdx.x * 16 + wave) * 2] = t0; ticks[(blockIdx.x * 16 + wave) * 2 + 1] = t1; }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0xdeadbeefu) sink[threadIdx.x] = acc.x;
}
template <int DW, int RW>
int run(const char* src, unsigned bytes, int mode, long long* dt, unsigned* sink, hipStream_t s) {
    const int iters = 400, grid = 256;
    auto kern = k<DW, RW>;
    CK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
    kern<<<grid, 64 * (DW + RW), 131072, s>>>(src, bytes, 20, mode, dt, sink);
    kern<<<grid, 64 * (DW + RW), 131072, s>>>(src, bytes, iters, mode, dt, sink);
    CK(hipStreamSynchronize(s));
    std::vector<long long> t(grid * 32);
    CK(hipMemcpy(t.data(), dt, grid * 32 * 8, hipMemcpyDeviceToHost));
    double sd = 0, sr = 0;
    for (int b = 0; b < grid; ++b) {
        for (int w = 0; w < DW; ++w) sd += t[(b * 16 + w) * 2 + 1] - t[(b * 16 + w) * 2];
        for (int w = DW; w < DW + RW; ++w) sr += t[(b * 16 + w) * 2 + 1] - t[(b * 16 + w) * 2];
    }
    sd /= grid * DW; sr /= grid * RW;
    printf("loaders %d readers %d mode %d: ", DW, RW, mode);
    if (mode & 1) printf("DMA %.1f B/tick/CU  ", (double)DW * 8192 * iters / sd);
    if (mode & 2) printf("reads %.1f B/tick/CU", (double)RW * 8192 * iters / sr);
    printf("\n");
    return 0;
}
int main() {
    hipStream_t s; CK(hipStreamCreate(&s));
    const unsigned bytes = 256u * 262144u;
    char* src; CK(hipMalloc(&src, bytes)); CK(hipMemset(src, 1, bytes));
    long long* dt; CK(hipMalloc(&dt, 256 * 32 * 8)); unsigned* sink; CK(hipMalloc(&sink, 8192));
    for (int mode : {1, 2, 3}) run<4, 4>(src, bytes, mode, dt, sink, s);
    for (int mode : {1, 2, 3}) run<4, 8>(src, bytes, mode, dt, sink, s);
    for (int mode : {1, 2, 3}) run<2, 8>(src, bytes, mode, dt, sink, s);
    return 0;
}
