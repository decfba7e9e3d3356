// Bandwidth-bound kernels of the EXEC path (input cast, pooling, FC, softmax) and the
// LOAD-time weight re-layout.  Activations are NHWC in the model's storage type.
#include "common.h"

namespace cw {

template <typename T>
static __device__ __forceinline__ float to_f32(T v) { return (float)v; }

// ---- input: fp32 NCHW [B][C][H][W] (C <= 4) -> NHWC4, channels C..3 zero ----------------
// One thread per pixel: C strided 4-byte reads (each coalesced across the wave along W), one
// 8-byte write.
template <typename T>
__global__ __launch_bounds__(256) void cast_input_kernel(const CastArgs a) {
    const size_t hw = (size_t)a.H * a.W;
    const size_t total = (size_t)a.B * hw;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const size_t n = i / hw, p = i - n * hw;
    T v[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] = (T)(c < a.C ? a.x[(n * a.C + c) * hw + p] : 0.f);
    *reinterpret_cast<uint2 *>(static_cast<T *>(a.y) + i * 4) = *reinterpret_cast<const uint2 *>(v);
}

// ---- max pool k x k, stride, pad (padded taps ignored); one thread = 8 channels ---------
template <typename T>
__global__ __launch_bounds__(256) void maxpool_kernel(const PoolArgs a) {
    const int c8 = a.C / 8;
    const size_t total = (size_t)a.B * a.Ho * a.Wo * c8;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int cg = (int)(i % c8);
    size_t t = i / c8;
    const int q = (int)(t % a.Wo);
    t /= a.Wo;
    const int p = (int)(t % a.Ho);
    const int n = (int)(t / a.Ho);
    float m[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) m[e] = -INFINITY;
    const T *xg = static_cast<const T *>(a.x);
    for (int r = 0; r < a.k; ++r) {
        const int ih = p * a.stride - a.pad + r;
        if ((unsigned)ih >= (unsigned)a.H) continue;
        for (int s = 0; s < a.k; ++s) {
            const int iw = q * a.stride - a.pad + s;
            if ((unsigned)iw >= (unsigned)a.W) continue;
            const uint4 raw = *reinterpret_cast<const uint4 *>(xg + (((size_t)n * a.H + ih) * a.W + iw) * a.C + cg * 8);
            const T *v = reinterpret_cast<const T *>(&raw);
#pragma unroll
            for (int e = 0; e < 8; ++e) m[e] = fmaxf(m[e], to_f32(v[e]));
        }
    }
    T out[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = (T)m[e];  // exact: the max is one of the inputs
    *reinterpret_cast<uint4 *>(static_cast<T *>(a.y) + i * 8) = *reinterpret_cast<const uint4 *>(out);
}

// ---- global average pool: NHWC [B][H*W][C] -> fp32 [B][C]; one thread = 8 channels ------
template <typename T>
__global__ __launch_bounds__(64) void gavgpool_kernel(const PoolArgs a) {
    const int c8 = a.C / 8;
    const int i = blockIdx.x * 64 + threadIdx.x;
    if (i >= a.B * c8) return;
    const int n = i / c8, cg = i - n * c8;
    const int hw = a.H * a.W;
    float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const T *xg = static_cast<const T *>(a.x) + (size_t)n * hw * a.C + cg * 8;
    for (int p = 0; p < hw; ++p) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(xg + (size_t)p * a.C);
        const T *v = reinterpret_cast<const T *>(&raw);
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] += to_f32(v[e]);
    }
    float *y = static_cast<float *>(a.y) + (size_t)n * a.C + cg * 8;
    const float inv = 1.f / (float)hw;
#pragma unroll
    for (int e = 0; e < 8; ++e) y[e] = s[e] * inv;
}

// ---- FC: z[n][j] = bias[j] + sum_i f[n][i] * W[j][i]; one wave per output j, up to 16 samples
// per launch row (blockIdx.y selects the group of 16 samples).  Weight streaming.
template <typename T>
__global__ __launch_bounds__(256) void fc_kernel(const FcArgs a) {
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= a.Out) return;  // whole wave exits together
    const int nb0 = blockIdx.y * 16;
    const int nb = min(16, a.B - nb0);
    float acc[16];
#pragma unroll
    for (int n = 0; n < 16; ++n) acc[n] = 0.f;
    const T *wrow = static_cast<const T *>(a.w) + (size_t)j * a.In;
    for (int i = lane * 8; i < a.In; i += 64 * 8) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(wrow + i);
        const T *wv = reinterpret_cast<const T *>(&raw);
        float wf[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) wf[e] = to_f32(wv[e]);
#pragma unroll
        for (int n = 0; n < 16; ++n) {
            if (n < nb) {
                const float4 f0 = *reinterpret_cast<const float4 *>(a.f + (size_t)(nb0 + n) * a.In + i);
                const float4 f1 = *reinterpret_cast<const float4 *>(a.f + (size_t)(nb0 + n) * a.In + i + 4);
                acc[n] += f0.x * wf[0] + f0.y * wf[1] + f0.z * wf[2] + f0.w * wf[3] +
                          f1.x * wf[4] + f1.y * wf[5] + f1.z * wf[6] + f1.w * wf[7];
            }
        }
    }
#pragma unroll
    for (int n = 0; n < 16; ++n) {
        float v = acc[n];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        if (lane == 0 && n < nb) a.z[(size_t)(nb0 + n) * a.Out + j] = v + a.bias[j];
    }
}

// ---- softmax over D values per row; one workgroup of 256 per row, wavefront reductions ---
__global__ __launch_bounds__(256) void softmax_kernel(const SoftmaxArgs a) {
    __shared__ float red[4];
    const int row = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *z = a.z + (size_t)row * a.D;
    float m = -INFINITY;
    for (int j = tid; j < a.D; j += 256) m = fmaxf(m, z[j]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if (lane == 0) red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float s = 0.f;
    for (int j = tid; j < a.D; j += 256) s += expf(z[j] - m);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) red[wave] = s;
    __syncthreads();
    s = (red[0] + red[1]) + (red[2] + red[3]);
    const float inv = 1.f / s;
    for (int j = tid; j < a.D; j += 256) a.p[(size_t)row * a.D + j] = expf(z[j] - m) * inv;
}

// ---- LOAD: canonical W[cout][cin][kh][kw] -> [cout][kh][kwp][cinp], zero padded ----------
// 16-bit elements are moved as raw bits, so one kernel serves fp16 and bf16.
__global__ __launch_bounds__(256) void pack_weights_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst,
                                                           int cout, int cin, int kh, int kw, int kwp, int cinp) {
    const size_t total = (size_t)cout * kh * kwp * cinp;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int c = (int)(i % cinp);
    size_t t = i / cinp;
    const int s = (int)(t % kwp);
    t /= kwp;
    const int r = (int)(t % kh);
    const int k = (int)(t / kh);
    uint16_t v = 0;
    if (c < cin && s < kw) v = src[(((size_t)k * cin + c) * kh + r) * kw + s];
    dst[i] = v;
}

__global__ __launch_bounds__(256) void copy_f32_kernel(const float *__restrict__ src, float *__restrict__ dst, size_t n) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint4 *dst, size_t n16) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n16; i += stride) dst[i] = make_uint4(0u, 0u, 0u, 0u);
}

template <typename T>
__global__ __launch_bounds__(256) void nhwc_to_nchw_f32_kernel(const T *__restrict__ src, float *__restrict__ dst,
                                                               int B, int C, int H, int W) {
    const size_t total = (size_t)B * C * H * W;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;  // NCHW index
    if (i >= total) return;
    const int w = (int)(i % W);
    size_t t = i / W;
    const int h = (int)(t % H);
    t /= H;
    const int c = (int)(t % C);
    const int n = (int)(t / C);
    dst[i] = (float)src[(((size_t)n * H + h) * W + w) * C + c];
}

static inline unsigned blocks_for(size_t n, int per) { return (unsigned)((n + per - 1) / per); }

#define CW_DISPATCH(dt, KERNEL, grid, block, s, ...)                   \
    do {                                                                \
        if ((dt) == DT_F16)                                             \
            KERNEL<f16><<<grid, block, 0, s>>>(__VA_ARGS__);            \
        else                                                            \
            KERNEL<bf16><<<grid, block, 0, s>>>(__VA_ARGS__);           \
    } while (0)

hipError_t launch_cast_input(DType dt, const CastArgs &a, hipStream_t s) {
    if (a.C < 1 || a.C > 4 || a.B < 1) return hipErrorInvalidValue;
    const size_t total = (size_t)a.B * a.H * a.W;
    CW_DISPATCH(dt, cast_input_kernel, dim3(blocks_for(total, 256)), 256, s, a);
    return hipGetLastError();
}

hipError_t launch_maxpool(DType dt, const PoolArgs &a, hipStream_t s) {
    if (a.C % 8 != 0 || a.B < 1) return hipErrorInvalidValue;
    const size_t total = (size_t)a.B * a.Ho * a.Wo * (a.C / 8);
    CW_DISPATCH(dt, maxpool_kernel, dim3(blocks_for(total, 256)), 256, s, a);
    return hipGetLastError();
}

hipError_t launch_gavgpool(DType dt, const PoolArgs &a, hipStream_t s) {
    if (a.C % 8 != 0 || a.B < 1) return hipErrorInvalidValue;
    const size_t total = (size_t)a.B * (a.C / 8);
    CW_DISPATCH(dt, gavgpool_kernel, dim3(blocks_for(total, 64)), 64, s, a);
    return hipGetLastError();
}

hipError_t launch_fc(DType dt, const FcArgs &a, hipStream_t s) {
    if (a.In % 512 != 0 || a.B < 1 || a.Out < 1) return hipErrorInvalidValue;
    const dim3 grid(blocks_for(a.Out, 4), blocks_for(a.B, 16));
    CW_DISPATCH(dt, fc_kernel, grid, 256, s, a);
    return hipGetLastError();
}

hipError_t launch_softmax(const SoftmaxArgs &a, hipStream_t s) {
    if (a.B < 1 || a.D < 1) return hipErrorInvalidValue;
    softmax_kernel<<<dim3(a.B), 256, 0, s>>>(a);
    return hipGetLastError();
}

hipError_t launch_pack_weights(const void *src, void *dst, int cout, int cin, int kh, int kw, int kwp, int cinp,
                               hipStream_t s) {
    const size_t total = (size_t)cout * kh * kwp * cinp;
    pack_weights_kernel<<<dim3(blocks_for(total, 256)), 256, 0, s>>>(static_cast<const uint16_t *>(src),
                                                                    static_cast<uint16_t *>(dst), cout, cin, kh, kw,
                                                                    kwp, cinp);
    return hipGetLastError();
}

hipError_t launch_copy_f32(const float *src, float *dst, size_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    copy_f32_kernel<<<dim3(blocks_for(n, 256)), 256, 0, s>>>(src, dst, n);
    return hipGetLastError();
}

hipError_t launch_fill_zero(void *dst, size_t bytes, hipStream_t s) {
    if (bytes % 16 != 0) return hipErrorInvalidValue;
    if (bytes == 0) return hipSuccess;
    const size_t n16 = bytes / 16;
    const unsigned grid = (unsigned)((n16 + 255) / 256 < 2048 ? (n16 + 255) / 256 : 2048);
    fill_zero_kernel<<<dim3(grid), 256, 0, s>>>(static_cast<uint4 *>(dst), n16);
    return hipGetLastError();
}

hipError_t launch_nhwc_to_nchw_f32(DType dt, const void *src, float *dst, int B, int C, int H, int W, hipStream_t s) {
    const size_t total = (size_t)B * C * H * W;
    if (dt == DT_F16)
        nhwc_to_nchw_f32_kernel<f16><<<dim3(blocks_for(total, 256)), 256, 0, s>>>(static_cast<const f16 *>(src), dst, B, C, H, W);
    else
        nhwc_to_nchw_f32_kernel<bf16><<<dim3(blocks_for(total, 256)), 256, 0, s>>>(static_cast<const bf16 *>(src), dst, B, C, H, W);
    return hipGetLastError();
}

}  // namespace cw
