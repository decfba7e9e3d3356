// Rate of direct-to-LDS buffer loads (buffer_load_dwordx4 ... lds) per compute unit, as the convolution
// kernel issues them: every workgroup streams tiles whose first part all workgroups share (weights,
// a 288 KiB region walked slice by slice) and whose rest is its own (activations, 64 KiB), all of it
// resident in L2 and far larger than the 32 KiB L1.  Prints bytes per shader clock per workgroup
// (one workgroup per CU up to 256 workgroups).  Stand-alone: hipcc --offload-arch=gfx950 -O3.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <algorithm>
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
// Each workgroup: `iters` rounds; per round each wave issues PER loads of 1 KiB covering
// a tile of WAVES*PER KiB. shared_bytes of the tile come from a region common to all workgroups,
// the rest from the workgroup's own region.  REG: 1 = loads to registers instead of LDS.
template <int WAVES, int PER, int REG>
__global__ __launch_bounds__(64 * WAVES) void k(const char* src, unsigned src_bytes, unsigned own_stride, unsigned shared_kib, int iters, long long* ticks, unsigned* sink) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const u32x4 d = make_desc(src, src_bytes);
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)lds;
    unsigned voff[PER]; bool is_shared[PER];
    const unsigned own_kib = WAVES * PER - shared_kib;
    for (int j = 0; j < PER; ++j) {
        const unsigned kib = wave * PER + j;   // which KiB of the tile
        voff[j] = (kib < shared_kib ? kib * 1024u : (1u << 20) + blockIdx.x * 65536u + (kib - shared_kib) * 1024u) + lane * 16u;
        is_shared[j] = kib < shared_kib;
    }
    u32x4 acc = {0, 0, 0, 0};
    __syncthreads();
    const long long t0 = clock64();
    unsigned so_sh = 0, so_own = 0;
    for (int it = 0; it < iters; ++it) {
        if (REG) {
            const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(src), 0, src_bytes, 0x00020000);
#pragma unroll
            for (int j = 0; j < PER; ++j) acc ^= __builtin_amdgcn_raw_buffer_load_b128(r, voff[j], is_shared[j] ? so_sh : so_own, 0);
        } else {
#pragma unroll
            for (int j = 0; j < PER; ++j) load_to_lds(d, voff[j], is_shared[j] ? so_sh : so_own, lds_base + (it & 1) * (WAVES * PER * 1024) + (wave * PER + j) * 1024u);
            asm volatile("s_waitcnt vmcnt(%0)" : : "n"(PER) : "memory");
        }
        // shared part walks a 288 KiB region (L2-resident, far larger than L1), own part a 64 KiB one
        so_sh += shared_kib * 1024u; if (so_sh + shared_kib * 1024u > 288u * 1024u) so_sh = 0;
        so_own += own_kib * 1024u; if (so_own + own_kib * 1024u > 65536u) so_own = 0;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const long long t1 = clock64();
    if (threadIdx.x == 0) { ticks[blockIdx.x * 2] = t0; ticks[blockIdx.x * 2 + 1] = t1; }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0xdeadbeefu) sink[threadIdx.x] = acc.x;
}
template <int WAVES, int PER, int REG>
int run(const char* src, unsigned src_bytes, int grid, unsigned shared_kib, long long* dt, unsigned* sink, hipStream_t s) {
    const int iters = 400;
    const unsigned tile = WAVES * PER * 1024;
    auto kern = k<WAVES, PER, REG>;
    CK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 2 * tile));
    kern<<<grid, 64 * WAVES, 2 * tile, s>>>(src, src_bytes, tile, shared_kib, 20, dt, sink);
    kern<<<grid, 64 * WAVES, 2 * tile, s>>>(src, src_bytes, tile, shared_kib, iters, dt, sink);
    CK(hipStreamSynchronize(s));
    std::vector<long long> t(grid * 2);
    CK(hipMemcpy(t.data(), dt, grid * 16, hipMemcpyDeviceToHost));
    double sum = 0; long long mx = 0;
    for (int b = 0; b < grid; ++b) { sum += t[2 * b + 1] - t[2 * b]; mx = std::max(mx, t[2 * b + 1] - t[2 * b]); }
    const double avg = sum / grid;
    printf("%s waves %d tile %3u KiB (shared %3u KiB) grid %4d: %.1f B/tick/WG avg (slowest WG %.1f)\n", REG ? "to-VGPR" : "to-LDS ", WAVES, tile / 1024, shared_kib, grid,
           (double)tile * iters / avg, (double)tile * iters / mx);
    return 0;
}
int main() {
    hipStream_t s; CK(hipStreamCreate(&s));
    const unsigned bytes = (1u << 20) + 1024u * 64 * 1024;   // 1 MiB shared region + 64 KiB per workgroup
    char* src; CK(hipMalloc(&src, bytes)); CK(hipMemset(src, 1, bytes));
    long long* dt; CK(hipMalloc(&dt, 1024 * 16)); unsigned* sink; CK(hipMalloc(&sink, 4096));
    for (int grid : {8, 128, 256, 512}) {
        run<4, 6, 0>(src, bytes, grid, 0, dt, sink, s);     // 24 KiB tiles, all own
        run<4, 6, 0>(src, bytes, grid, 16, dt, sink, s);    // 16 KiB shared (weights) + 8 own
        run<8, 3, 0>(src, bytes, grid, 16, dt, sink, s);
        run<4, 6, 1>(src, bytes, grid, 16, dt, sink, s);    // the same bytes into registers
    }
    run<4, 8, 0>(src, bytes, 256, 16, dt, sink, s);
    run<4, 16, 0>(src, bytes, 256, 32, dt, sink, s);
    run<8, 8, 0>(src, bytes, 256, 32, dt, sink, s);
    run<16, 4, 0>(src, bytes, 256, 32, dt, sink, s);
    return 0;
}
