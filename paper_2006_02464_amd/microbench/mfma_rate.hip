// Issue rate of v_mfma_f32_32x32x16_f16 and v_mfma_f32_16x16x32_f16: shader clocks per instruction per
// wave for 1, 2, 4 or 8 independent accumulators (1 = every MFMA depends on the one before), with 1, 2
// and 4 waves per SIMD, and the resulting TFLOP/s of the whole chip.  Stand-alone:
// hipcc --offload-arch=gfx950 -O3.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
typedef _Float16 v8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
template <int KIND, int CHAINS>
__global__ void k(int iters, long long* ticks, float* sink) {
    v8 a, b;
    for (int e = 0; e < 8; ++e) { a[e] = (_Float16)(threadIdx.x * 0.001f + e); b[e] = (_Float16)(e * 0.5f); }
    f32x16 acc[CHAINS]; f32x4 acc4[CHAINS];
    for (int c = 0; c < CHAINS; ++c) { for (int e = 0; e < 16; ++e) acc[c][e] = 0.f; for (int e = 0; e < 4; ++e) acc4[c][e] = 0.f; }
    __syncthreads();
    const long long t0 = clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < CHAINS; ++c) {
            if (KIND == 0) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[c], 0, 0, 0);
            else acc4[c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc4[c], 0, 0, 0);
        }
    }
    float s = 0.f;
    for (int c = 0; c < CHAINS; ++c) { for (int e = 0; e < 16; ++e) s += acc[c][e]; for (int e = 0; e < 4; ++e) s += acc4[c][e]; }
    const long long t1 = clock64();
    if ((threadIdx.x & 63) == 0) { ticks[(blockIdx.x * 16 + (threadIdx.x >> 6)) * 2] = t0; ticks[(blockIdx.x * 16 + (threadIdx.x >> 6)) * 2 + 1] = t1; }
    if (s == 123.456f) sink[threadIdx.x] = s;
}
template <int KIND, int CHAINS>
int run(int waves, long long* dt, float* sink) {
    const int iters = 2000, grid = 256;
    k<KIND, CHAINS><<<grid, 64 * waves>>>(10, dt, sink);
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    CK(hipEventRecord(e0, 0));
    k<KIND, CHAINS><<<grid, 64 * waves>>>(iters, dt, sink);
    CK(hipEventRecord(e1, 0));
    CK(hipDeviceSynchronize());
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    std::vector<long long> t(grid * 32);
    CK(hipMemcpy(t.data(), dt, grid * 32 * 8, hipMemcpyDeviceToHost));
    double sum = 0;
    for (int b = 0; b < grid; ++b) for (int w = 0; w < waves; ++w) sum += t[(b * 16 + w) * 2 + 1] - t[(b * 16 + w) * 2];
    const double per_wave = sum / (grid * waves) / ((double)iters * CHAINS);
    const double flops = (KIND == 0 ? 32768.0 : 16384.0) * iters * CHAINS * waves * grid;
    printf("%s accumulators %d waves/CU %2d: %.1f clocks per MFMA per wave; kernel %.3f ms -> %.0f TFLOP/s\n", KIND == 0 ? "32x32x16" : "16x16x32", CHAINS, waves,
           per_wave, ms, flops / (ms * 1e-3) / 1e12);
    return 0;
}
int main() {
    long long* dt; CK(hipMalloc(&dt, 256 * 32 * 8)); float* sink; CK(hipMalloc(&sink, 4096));
    run<0, 1>(4, dt, sink); run<0, 2>(4, dt, sink); run<0, 4>(4, dt, sink); run<0, 4>(8, dt, sink); run<0, 4>(16, dt, sink);
    run<1, 1>(4, dt, sink); run<1, 4>(4, dt, sink); run<1, 8>(4, dt, sink); run<1, 8>(8, dt, sink);
    return 0;
}
