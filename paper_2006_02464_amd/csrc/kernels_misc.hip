// Bandwidth-bound kernels of the EXEC path (input cast, pooling, FC, softmax) and the
// LOAD-time weight re-layout.  Activations are NHWC in the model's storage type.
#include "common.h"
#include "conv_common.h"

namespace cw {

// The kernels of EXEC take their arguments as scalars, not as a struct: this file is compiled with
// kernel-argument preloading, so up to 14 dwords of them are in SGPRs when a wave starts.
template <typename T>
static __device__ __forceinline__ float to_f32(T v) { return (float)v; }

// ---- input: fp32 NCHW [B][C][H][W] (C <= 4) -> NHWC4, channels C..3 zero ----------------
// One thread per pixel of the padded output: inside the image C strided 4-byte reads (each
// coalesced across the wave along W), zeros in the border; one 8-byte write either way.
template <typename T>
__global__ __launch_bounds__(256) void cast_input_kernel(const float *x, void *y, int B, int C, int H, int W, int pad, int Hp, int Wp) {
    const CastArgs a{x, y, B, C, H, W, pad, Hp, Wp};
    // 32-bit index arithmetic: the launch code checks that the padded output has fewer than 2^31 pixels
    const unsigned hwp = (unsigned)a.Hp * a.Wp;
    const unsigned total = (unsigned)a.B * hwp;
    const unsigned i = blockIdx.x * 256u + threadIdx.x;
    if (i >= total) return;
    const unsigned n = i / hwp, pp = i - n * hwp;
    const unsigned row = pp / (unsigned)a.Wp;
    const int ih = (int)row - a.pad, iw = (int)(pp - row * (unsigned)a.Wp) - a.pad;
    T v[4] = {(T)0.f, (T)0.f, (T)0.f, (T)0.f};
    if ((unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W) {
        const size_t hw = (size_t)a.H * a.W, p = (size_t)ih * a.W + iw;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (c < a.C) v[c] = (T)a.x[((size_t)n * a.C + c) * hw + p];
    }
    *reinterpret_cast<uint2 *>(static_cast<T *>(a.y) + (size_t)i * 4) = *reinterpret_cast<const uint2 *>(v);
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

// Workgroups go to the 8 XCDs in turn.  Kernels whose neighbouring workgroups read overlapping
// windows number their blocks so that each XCD computes one contiguous eighth of the output, and
// the overlap is found in that XCD's L2 instead of being fetched once per XCD.
static __device__ __forceinline__ unsigned xcd_block(unsigned bid, unsigned nb) {
    const unsigned xcd = bid & 7u, idx = bid >> 3;
    const unsigned per = nb >> 3, rem = nb & 7u;
    return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}

// The same for a window of KS x KS known at compile time and fewer than 2^31 elements: the KS*KS
// loads of a thread do not depend on each other and are requested together (out-of-range taps read
// a clamped, valid address and are not counted), and the index arithmetic is 32-bit.
template <typename T, int KS>
__global__ __launch_bounds__(256) void maxpool_window_kernel(const void *x, void *y, int B, int H, int W, int C, int Ho, int Wo, int k, int stride, int pad) {
    const PoolArgs a{x, y, B, H, W, C, Ho, Wo, k, stride, pad};
    const unsigned c8 = (unsigned)a.C / 8u;
    const unsigned total = (unsigned)a.B * a.Ho * a.Wo * c8;
    const unsigned i = xcd_block(blockIdx.x, gridDim.x) * 256u + threadIdx.x;
    if (i >= total) return;
    const unsigned cg = i % c8;
    unsigned t = i / c8;
    const int q = (int)(t % (unsigned)a.Wo);
    t /= (unsigned)a.Wo;
    const int p = (int)(t % (unsigned)a.Ho);
    const unsigned n = t / (unsigned)a.Ho;
    const T *xg = static_cast<const T *>(a.x) + (size_t)n * a.H * a.W * a.C + cg * 8u;
    uint4 raw[KS * KS];
    bool ok[KS * KS];
#pragma unroll
    for (int r = 0; r < KS; ++r)
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int ih = p * a.stride - a.pad + r, iw = q * a.stride - a.pad + s;
            ok[r * KS + s] = (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
            const unsigned ihc = (unsigned)min(max(ih, 0), a.H - 1), iwc = (unsigned)min(max(iw, 0), a.W - 1);
            raw[r * KS + s] = *reinterpret_cast<const uint4 *>(xg + (ihc * (unsigned)a.W + iwc) * (unsigned)a.C);
        }
    float m[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) m[e] = -INFINITY;
#pragma unroll
    for (int k = 0; k < KS * KS; ++k) {
        const T *v = reinterpret_cast<const T *>(&raw[k]);
#pragma unroll
        for (int e = 0; e < 8; ++e) m[e] = ok[k] ? fmaxf(m[e], to_f32(v[e])) : m[e];
    }
    T out[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = (T)m[e];  // exact: the max is one of the inputs
    *reinterpret_cast<uint4 *>(static_cast<T *>(a.y) + (size_t)i * 8) = *reinterpret_cast<const uint4 *>(out);
}

// ---- max pool and the 1x1 convolution that reads it, in one launch -----------------------
// A workgroup of 4 waves takes BM pooled pixels x 64 channels: every thread computes BM/32 pieces
// (pixel, 8 channels) of the pooled tile as the kernel above does, writes them to the pooled tensor
// (its other readers need it) and into LDS in the convolution kernel's operand layout (128-byte
// rows, 16-byte chunks swizzled); the N x 64 weights (N = 64 or 128) go to LDS the same way.  After one barrier the
// waves (2 x 2 over pixels x output channels) run the 64-deep product on the matrix cores, in the
// same k order as the convolution kernel, and store through its epilogue (bias, activation, one
// rounding).  The 1x1 convolution then costs no launch of its own and never reads its input from memory.
template <typename T, int KS, int BM, int N>
__global__ __launch_bounds__(256) void maxpool_conv1x1_kernel(const PoolArgs a, const ConvArgs c) {
    constexpr int C = 64;                // channels of the pooled tensor; N = output channels of the convolution
    constexpr int PIECES = BM * (C / 8) / 256;
    constexpr int TM = BM / 64, TN = N / 64;
    typedef typename Mfma<T>::v8 v8;
    __shared__ __attribute__((aligned(16))) T sX[BM * C];
    __shared__ __attribute__((aligned(16))) T sW[N * C];
    const unsigned tid = threadIdx.x;
    const unsigned m0 = xcd_block(blockIdx.x, gridDim.x) * (unsigned)BM;
    const unsigned M = (unsigned)a.B * a.Ho * a.Wo;
    const int lane = tid & 63, wave = tid >> 6;
    const EpiPos pos{(int)m0, 0, (wave >> 1) * (BM / 2), (wave & 1) * (N / 2), lane & 31, lane >> 5};
    EpiOperands<TM, TN> eo;
    epilogue_load<TM, TN>(eo, c, pos);   // the bias, requested beside the window loads
    uint4 wraw[N * (C / 8) / 256];       // N x 64 weights: row = output channel
#pragma unroll
    for (int j = 0; j < N * (C / 8) / 256; ++j) {
        const unsigned cid = tid + j * 256u;
        wraw[j] = *reinterpret_cast<const uint4 *>(static_cast<const T *>(c.w) + (cid >> 3) * C + (cid & 7u) * 8u);
    }
    uint4 raw[PIECES][KS * KS];
    bool ok[PIECES][KS * KS];
#pragma unroll
    for (int j = 0; j < PIECES; ++j) {
        const unsigned cid = tid + j * 256u;
        const unsigned m = min(m0 + (cid >> 3), M - 1u), cg = cid & 7u;   // rows beyond M: a valid pixel, not stored
        unsigned t = m / (unsigned)a.Wo;
        const int q = (int)(m - t * (unsigned)a.Wo);
        const unsigned n = t / (unsigned)a.Ho;
        const int p = (int)(t - n * (unsigned)a.Ho);
        const T *xg = static_cast<const T *>(a.x) + (size_t)n * a.H * a.W * C + cg * 8u;
#pragma unroll
        for (int r = 0; r < KS; ++r)
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const int ih = p * a.stride - a.pad + r, iw = q * a.stride - a.pad + s;
                ok[j][r * KS + s] = (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
                const unsigned ihc = (unsigned)min(max(ih, 0), a.H - 1), iwc = (unsigned)min(max(iw, 0), a.W - 1);
                raw[j][r * KS + s] = *reinterpret_cast<const uint4 *>(xg + (ihc * (unsigned)a.W + iwc) * (unsigned)C);
            }
    }
#pragma unroll
    for (int j = 0; j < N * (C / 8) / 256; ++j) {
        const unsigned cid = tid + j * 256u;
        *reinterpret_cast<uint4 *>(sW + swz<C>((int)(cid >> 3), (int)(cid & 7u))) = wraw[j];
    }
#pragma unroll
    for (int j = 0; j < PIECES; ++j) {
        const unsigned cid = tid + j * 256u;
        const unsigned row = cid >> 3, cg = cid & 7u;
        float mx[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) mx[e] = -INFINITY;
#pragma unroll
        for (int k = 0; k < KS * KS; ++k) {
            const T *v = reinterpret_cast<const T *>(&raw[j][k]);
#pragma unroll
            for (int e = 0; e < 8; ++e) mx[e] = ok[j][k] ? fmaxf(mx[e], to_f32(v[e])) : mx[e];
        }
        T out[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = (T)mx[e];  // exact: the max is one of the inputs
        const uint4 o = *reinterpret_cast<const uint4 *>(out);
        if (m0 + row < M) *reinterpret_cast<uint4 *>(static_cast<T *>(a.y) + ((size_t)(m0 + row) * C + cg * 8u)) = o;
        *reinterpret_cast<uint4 *>(sX + swz<C>((int)row, (int)cg)) = o;   // rows beyond M hold a copy of the last pixel; never stored
    }
    __syncthreads();
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
#pragma unroll
    for (int kk = 0; kk < C / 16; ++kk) {
        v8 fw[TN], fx[TM];
#pragma unroll
        for (int j = 0; j < TN; ++j) fw[j] = *reinterpret_cast<const v8 *>(sW + swz<C>(pos.wn0 + j * 32 + pos.lrow, kk * 2 + pos.lhalf));
#pragma unroll
        for (int i = 0; i < TM; ++i) fx[i] = *reinterpret_cast<const v8 *>(sX + swz<C>(pos.wm0 + i * 32 + pos.lrow, kk * 2 + pos.lhalf));
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = Mfma<T>::mma(fw[j], fx[i], acc[i][j]);
    }
    epilogue_store<T, TM, TN>(acc, eo, c, pos);
}

// ---- global average pool: NHWC [B][H*W][C] -> fp32 [B][C] -------------------------------
// One wave per (sample, 64 channels): lane = (part, group) with group = lane%8 owning 8
// channels and part = lane/8 taking pixels part, part+8, ...; the 8 parts are then summed with
// three xor-shuffles in a fixed order.  8 lanes read one pixel's 128 contiguous bytes.
template <typename T>
__global__ __launch_bounds__(64) void gavgpool_kernel(const void *x, void *y, int B, int H, int W, int C, int Ho, int Wo, int k, int stride, int pad) {
    const PoolArgs a{x, y, B, H, W, C, Ho, Wo, k, stride, pad};
    const int groups = a.C / 64;
    const int n = blockIdx.x / groups, cb = (blockIdx.x - n * groups) * 64;
    const int lane = threadIdx.x, cg = lane & 7, part = lane >> 3;
    const int hw = a.H * a.W;
    float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const T *xg = static_cast<const T *>(a.x) + (size_t)n * hw * a.C + cb + cg * 8;
    // rounds of 8 pixels per lane, their loads requested together (a 7x7 map is one round); a pixel
    // past the end reads the last one and is not added
    for (int p0 = part; p0 < hw; p0 += 64) {
        uint4 raw[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) raw[u] = *reinterpret_cast<const uint4 *>(xg + (size_t)min(p0 + 8 * u, hw - 1) * a.C);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const T *v = reinterpret_cast<const T *>(&raw[u]);
            const bool live = p0 + 8 * u < hw;
#pragma unroll
            for (int e = 0; e < 8; ++e) s[e] += live ? to_f32(v[e]) : 0.f;
        }
    }
#pragma unroll
    for (int off = 8; off < 64; off <<= 1)
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] += __shfl_xor(s[e], off, 64);
    if (part == 0) {
        float *y = static_cast<float *>(a.y) + (size_t)n * a.C + cb + cg * 8;
        const float inv = 1.f / (float)hw;
        *reinterpret_cast<float4 *>(y) = make_float4(s[0] * inv, s[1] * inv, s[2] * inv, s[3] * inv);
        *reinterpret_cast<float4 *>(y + 4) = make_float4(s[4] * inv, s[5] * inv, s[6] * inv, s[7] * inv);
    }
}

// The same for large maps (hundreds of pixels and more: the DenseNet- and Inception-style lists pool
// 28x28 and 56x56 maps): kGapWaves waves per (sample, 64 channels); wave w takes the rounds w,
// w + kGapWaves, ... of 64 pixels; the waves' sums meet in LDS and are added in wave order.
constexpr int kGapWaves = 16;
template <typename T>
__global__ __launch_bounds__(64 * kGapWaves) void gavgpool_wide_kernel(const void *x, void *y, int B, int H, int W, int C, int Ho, int Wo, int k, int stride, int pad) {
    const PoolArgs a{x, y, B, H, W, C, Ho, Wo, k, stride, pad};
    __shared__ float red[kGapWaves][8][8];
    const int groups = a.C / 64;
    const int n = blockIdx.x / groups, cb = (blockIdx.x - n * groups) * 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, cg = lane & 7, part = lane >> 3;
    const int hw = a.H * a.W;
    float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const T *xg = static_cast<const T *>(a.x) + (size_t)n * hw * a.C + cb + cg * 8;
    for (int p0 = part + 64 * wave; p0 < hw; p0 += 64 * kGapWaves) {
        uint4 raw[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) raw[u] = *reinterpret_cast<const uint4 *>(xg + (size_t)min(p0 + 8 * u, hw - 1) * a.C);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const T *v = reinterpret_cast<const T *>(&raw[u]);
            const bool live = p0 + 8 * u < hw;
#pragma unroll
            for (int e = 0; e < 8; ++e) s[e] += live ? to_f32(v[e]) : 0.f;
        }
    }
#pragma unroll
    for (int off = 8; off < 64; off <<= 1)
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] += __shfl_xor(s[e], off, 64);
    if (part == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) red[wave][cg][e] = s[e];
    }
    __syncthreads();
    if (threadIdx.x < 64) {   // 8 channel groups x 8 channels
        const int g = threadIdx.x >> 3, e = threadIdx.x & 7;
        float t = red[0][g][e];
#pragma unroll
        for (int w = 1; w < kGapWaves; ++w) t += red[w][g][e];
        static_cast<float *>(a.y)[(size_t)n * a.C + cb + g * 8 + e] = t * (1.f / (float)hw);
    }
}

// ---- FC: z[n][j] = bias[j] + sum_i f[n][i] * W[j][i], fp32 features, fp32 result ---------
// A workgroup computes 16 outputs x 16 samples on the matrix cores (v_mfma_f32_16x16x32 in the
// storage type: 16 output rows x 16 sample columns x 32 k per instruction).  Its 8 waves split K;
// wave w walks chunks of 32 k: lane (r = lane%16, g = lane/16) loads 8 consecutive weights of
// output row r and 8 consecutive features of sample r, both at k = chunk + 8g.  The layer streams
// its weights once from HBM, so the loads of four chunks are requested together before their 32
// MFMAs: the memory latency is paid once per 128 k, not once per chunk.  The eight partial
// 16x16 tiles are summed through LDS in wave order, the bias is added and the logits written.
typedef float fc_f32x4 __attribute__((ext_vector_type(4)));
constexpr int kFcWaves = 8;
template <typename T>
struct FcMfma;
template <>
struct FcMfma<f16> {
    typedef _Float16 elem;
    typedef _Float16 v8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ fc_f32x4 mma(v8 rows, v8 cols, fc_f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(rows, cols, c, 0, 0, 0); }
};
template <>
struct FcMfma<bf16> {
    typedef __bf16 elem;
    typedef __bf16 v8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ fc_f32x4 mma(v8 rows, v8 cols, fc_f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(rows, cols, c, 0, 0, 0); }
};

template <typename T>
__global__ __launch_bounds__(64 * kFcWaves) void fc_kernel(const float *f, const void *w, const float *bias, float *z, int B, int In, int Out) {
    const FcArgs a{f, w, bias, z, B, In, Out};
    __shared__ float part[kFcWaves][16][17];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int j = blockIdx.x * 16 + r;   // output row this lane feeds
    const int n = blockIdx.y * 16 + r;   // sample column this lane feeds
    const bool j_ok = j < a.Out, n_ok = n < a.B;
    const T *wrow = static_cast<const T *>(a.w) + (size_t)(j_ok ? j : 0) * a.In;
    const float *frow = a.f + (size_t)(n_ok ? n : 0) * a.In;
    fc_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const int kq = a.In / kFcWaves;  // K range of this wave (a multiple of 32)
    const int k_end = (wave + 1) * kq;
    for (int k0 = wave * kq + g * 8; k0 < k_end; k0 += 128) {
        uint4 wraw[4];
        float4 f0[4], f1[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int k = k0 + 32 * u;
            const bool live = k < k_end;  // uniform per wave
            const int kc = live ? k : k0;
            wraw[u] = *reinterpret_cast<const uint4 *>(wrow + kc);
            f0[u] = *reinterpret_cast<const float4 *>(frow + kc);
            f1[u] = *reinterpret_cast<const float4 *>(frow + kc + 4);
            if (!j_ok || !live) wraw[u] = make_uint4(0u, 0u, 0u, 0u);
            if (!n_ok) { f0[u] = make_float4(0.f, 0.f, 0.f, 0.f); f1[u] = f0[u]; }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            // 16x16x32 MFMA in the storage type: the lane's 8 weights and 8 features are exactly its
            // operand fragments (row/column lane%16, k = 8*(lane/16)..+7).  The fp32 features are
            // split into a storage-type head and the rounding remainder, two MFMAs per chunk, so
            // nothing of the fp32 value is lost beyond the remainder's own rounding (2^-22 relative
            // for fp16, 2^-17 for bf16).
            const float fv[8] = {f0[u].x, f0[u].y, f0[u].z, f0[u].w, f1[u].x, f1[u].y, f1[u].z, f1[u].w};
            typename FcMfma<T>::v8 hi, lo;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                hi[e] = (typename FcMfma<T>::elem)fv[e];
                lo[e] = (typename FcMfma<T>::elem)(fv[e] - (float)hi[e]);
            }
            const typename FcMfma<T>::v8 wv = *reinterpret_cast<const typename FcMfma<T>::v8 *>(&wraw[u]);
            acc = FcMfma<T>::mma(wv, hi, acc);
            acc = FcMfma<T>::mma(wv, lo, acc);
        }
    }
    // lane holds column (sample) lane%16, rows (outputs) 4*(lane/16) + e
#pragma unroll
    for (int e = 0; e < 4; ++e) part[wave][4 * g + e][r] = acc[e];
    __syncthreads();
    const int t = threadIdx.x;
    if (t < 256) {  // 16 outputs x 16 samples
        const int oj = t >> 4, on = t & 15;
        const int jj = blockIdx.x * 16 + oj, nn = blockIdx.y * 16 + on;
        if (jj < a.Out && nn < a.B) {
            float v = part[0][oj][on];
#pragma unroll
            for (int w = 1; w < kFcWaves; ++w) v += part[w][oj][on];
            a.z[(size_t)nn * a.Out + jj] = v + a.bias[jj];
        }
    }
}

// FC and softmax as one launch, for at most 16 samples and 1024 classes.  Grid (16-output tiles,
// K splits): a workgroup of 4 waves computes a 16 x 16 partial tile over In / split_k of K (each wave
// a quarter of that, chunks as above).  The splits of a tile meet like the convolution's split-K:
// partial tiles go to memory with device-scope stores, a ticket per tile makes the last arrival add
// them in split order, so the logits do not depend on arrival order.  A second ticket over the
// tiles makes the workgroup that completes the last tile compute the softmax of every row (wave w
// takes rows w, w+4, ...: a row is 16 values per lane, max and sum by wave shuffles; the same
// formula as the stand-alone kernels), so no second launch and no second pass over the logits.
// Workgroups sit on different XCDs: everything another workgroup reads travels device-scope.
constexpr int kFcsWaves = 4;
template <typename T>
__global__ __launch_bounds__(64 * kFcsWaves) void fc_softmax_kernel(const float *f, const void *w, const float *bias, float *z, float *p,
                                                                    float *partial, int *counters, int B, int In, int Out, int S) {
    __shared__ float part[kFcsWaves][16][17];
    __shared__ int s_last;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int j = blockIdx.x * 16 + r;   // output row this lane feeds
    const bool j_ok = j < Out, n_ok = r < B;
    const T *wrow = static_cast<const T *>(w) + (size_t)(j_ok ? j : 0) * In;
    const float *frow = f + (size_t)(n_ok ? r : 0) * In;
    fc_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const int kq = In / (kFcsWaves * S);  // K range of this wave (a multiple of 32)
    const int k_begin = ((int)blockIdx.y * kFcsWaves + wave) * kq, k_end = k_begin + kq;
    for (int k0 = k_begin + g * 8; k0 < k_end; k0 += 128) {
        uint4 wraw[4];
        float4 f0[4], f1[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int k = k0 + 32 * u;
            const bool live = k < k_end;  // uniform per wave
            const int kc = live ? k : k0;
            wraw[u] = *reinterpret_cast<const uint4 *>(wrow + kc);
            f0[u] = *reinterpret_cast<const float4 *>(frow + kc);
            f1[u] = *reinterpret_cast<const float4 *>(frow + kc + 4);
            if (!j_ok || !live) wraw[u] = make_uint4(0u, 0u, 0u, 0u);
            if (!n_ok) { f0[u] = make_float4(0.f, 0.f, 0.f, 0.f); f1[u] = f0[u]; }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float fv[8] = {f0[u].x, f0[u].y, f0[u].z, f0[u].w, f1[u].x, f1[u].y, f1[u].z, f1[u].w};
            typename FcMfma<T>::v8 hi, lo;   // fp32 feature = storage-type head + rounding remainder, as in fc_kernel
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                hi[e] = (typename FcMfma<T>::elem)fv[e];
                lo[e] = (typename FcMfma<T>::elem)(fv[e] - (float)hi[e]);
            }
            const typename FcMfma<T>::v8 wv = *reinterpret_cast<const typename FcMfma<T>::v8 *>(&wraw[u]);
            acc = FcMfma<T>::mma(wv, hi, acc);
            acc = FcMfma<T>::mma(wv, lo, acc);
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) part[wave][4 * g + e][r] = acc[e];
    __syncthreads();
    const int t = threadIdx.x;           // 256 threads = 16 outputs x 16 samples
    const int oj = t >> 4, on = t & 15;
    const int jj = blockIdx.x * 16 + oj;
    const bool live = jj < Out && on < B;
    float v = (part[0][oj][on] + part[1][oj][on]) + (part[2][oj][on] + part[3][oj][on]);
    if (S > 1) {
        if (live) __hip_atomic_store(&partial[((size_t)blockIdx.y * 16 + on) * Out + jj], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_s_waitcnt(0);   // this thread's partial sum has been written
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();                 // ... and so have the workgroup's
        if (t == 0) {
            const int ticket = __hip_atomic_fetch_add(&counters[blockIdx.x], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int last = ticket == S - 1;
            if (last) __hip_atomic_store(&counters[blockIdx.x], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next launch
            s_last = last;
        }
        __syncthreads();
        if (!s_last) return;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        v = 0.f;
        if (live)
            for (int s = 0; s < S; ++s)
                v += __hip_atomic_load(&partial[((size_t)s * 16 + on) * Out + jj], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (live) __hip_atomic_store(&z[(size_t)on * Out + jj], v + bias[jj], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // ---- the workgroup that completes the last tile turns the logits into probabilities
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (t == 0) {
        int *all = counters + gridDim.x;
        const int ticket = __hip_atomic_fetch_add(all, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = ticket == (int)gridDim.x - 1;
        if (last) __hip_atomic_store(all, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = last;
    }
    __syncthreads();
    if (!s_last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    constexpr int PER = kFcSoftmaxMaxOut / 64, ROWS = kFcSoftmaxMaxBatch / kFcsWaves;
    float vals[ROWS][PER];
#pragma unroll
    for (int q = 0; q < ROWS; ++q) {
        const int row = wave + kFcsWaves * q;
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            const int c = lane + 64 * e;
            vals[q][e] = (row < B && c < Out) ? __hip_atomic_load(&z[(size_t)row * Out + c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : -INFINITY;
        }
    }
#pragma unroll
    for (int q = 0; q < ROWS; ++q) {
        const int row = wave + kFcsWaves * q;
        if (row >= B) continue;   // uniform per wave
        float m = vals[q][0];
#pragma unroll
        for (int e = 1; e < PER; ++e) m = fmaxf(m, vals[q][e]);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
        float sum = 0.f;
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            vals[q][e] = expf(vals[q][e] - m);   // classes past Out: exp(-inf) = 0
            sum += vals[q][e];
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
        const float inv = 1.f / sum;
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            const int c = lane + 64 * e;
            if (c < Out) p[(size_t)row * Out + c] = vals[q][e] * inv;
        }
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

// The same for rows of at most 256 * PER values: a thread keeps its values j = tid, tid + 256, ... in
// registers, so a row is read once and every exponential computed once.  Same formula, same order of
// every sum as softmax_kernel: the results are identical.
template <int PER>
__global__ __launch_bounds__(256) void softmax_rows_kernel(const float *z_in, float *p_out, int B, int D) {
    const SoftmaxArgs a{z_in, p_out, B, D};
    __shared__ float red_m[4], red_s[4];
    const int row = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *z = a.z + (size_t)row * a.D;
    float v[PER];
    float m = -INFINITY;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int j = tid + e * 256;
        v[e] = j < a.D ? z[j] : -INFINITY;
        m = fmaxf(m, v[e]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if (lane == 0) red_m[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int j = tid + e * 256;
        if (j < a.D) {
            v[e] = expf(v[e] - m);
            s += v[e];
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) red_s[wave] = s;
    __syncthreads();
    s = (red_s[0] + red_s[1]) + (red_s[2] + red_s[3]);
    const float inv = 1.f / s;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int j = tid + e * 256;
        if (j < a.D) a.p[(size_t)row * a.D + j] = v[e] * inv;
    }
}

// ---- LOAD: canonical W[cout][cin][kh][kw] -> [cout'][kh][kwp][cinp], zero padded ---------
// 16-bit elements are moved as raw bits, so one kernel serves fp16 and bf16.  With `permute`,
// ---- depthwise convolution: one kh x kw filter per channel; one thread = 8 channels of one
// output pixel.  The bytes moved are the bound (one multiply-add per 2 bytes read at 3x3 stride 1);
// neighbouring threads cover neighbouring channel groups, so every access of a wave is one run of
// 16-byte pieces, and the taps' overlap between neighbouring pixels is served by the caches.
// Weights are [kh][kw][C] in the storage type; fp32 accumulation; + bias, + residual, activation,
// one round-to-nearest-even; x and y may be channel ranges of wider tensors (ldx, ldy).
static __device__ __forceinline__ float dw_act(float v, int act) {
    const float r = fmaxf(v, 0.f);
    const float h = v * fminf(fmaxf(v + 3.f, 0.f), 6.f) * (1.f / 6.f);
    return act == ACT_RELU ? r : (act == ACT_HSWISH ? h : v);
}

template <typename T>
__global__ __launch_bounds__(256) void dwconv_kernel(const DwArgs a) {
    const unsigned c8 = (unsigned)a.C / 8u;
    const unsigned total = (unsigned)a.B * a.Ho * a.Wo * c8;   // < 2^31: checked by the launch code
    const unsigned i = xcd_block(blockIdx.x, gridDim.x) * 256u + threadIdx.x;
    if (i >= total) return;
    const unsigned cg = i % c8;
    unsigned t = i / c8;            // output pixel m
    const unsigned m = t;
    const int q = (int)(t % (unsigned)a.Wo);
    t /= (unsigned)a.Wo;
    const int p = (int)(t % (unsigned)a.Ho);
    const unsigned n = t / (unsigned)a.Ho;
    float acc[8];
    {
        const float4 b0 = *reinterpret_cast<const float4 *>(a.bias + cg * 8u);
        const float4 b1 = *reinterpret_cast<const float4 *>(a.bias + cg * 8u + 4u);
        acc[0] = b0.x; acc[1] = b0.y; acc[2] = b0.z; acc[3] = b0.w;
        acc[4] = b1.x; acc[5] = b1.y; acc[6] = b1.z; acc[7] = b1.w;
    }
    const T *x = static_cast<const T *>(a.x);
    const T *w = static_cast<const T *>(a.w);
    for (int r = 0; r < a.kh; ++r) {
        const int ih = p * a.stride - a.pad + r;
        if ((unsigned)ih >= (unsigned)a.H) continue;
        for (int s = 0; s < a.kw; ++s) {
            const int iw = q * a.stride - a.pad + s;
            if ((unsigned)iw >= (unsigned)a.W) continue;
            const uint4 xv = *reinterpret_cast<const uint4 *>(x + ((size_t)(n * a.H + ih) * a.W + iw) * a.ldx + cg * 8u);
            const uint4 wv = *reinterpret_cast<const uint4 *>(w + (size_t)(r * a.kw + s) * a.C + cg * 8u);
            const T *xe = reinterpret_cast<const T *>(&xv);
            const T *we = reinterpret_cast<const T *>(&wv);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += (float)xe[e] * (float)we[e];
        }
    }
    if (a.res) {
        const uint4 rv = *reinterpret_cast<const uint4 *>(static_cast<const T *>(a.res) + (size_t)m * a.C + cg * 8u);
        const T *re = reinterpret_cast<const T *>(&rv);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += (float)re[e];
    }
    T out[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = (T)dw_act(acc[e], a.act);
    *reinterpret_cast<uint4 *>(static_cast<T *>(a.y) + (size_t)m * a.ldy + cg * 8u) = *reinterpret_cast<const uint4 *>(out);
}

// ---- depthwise 3x3 convolution and the 1x1 convolution that reads it, in one launch --------
// (a depthwise-separable block.)  A workgroup of 4 waves takes BM output pixels: every thread computes
// BM*C/2048 pieces (pixel, 8 channels) of the depthwise result, their loads requested together, exactly as
// dwconv_kernel does (bias first, the
// taps in filter order, fp32, activation, one rounding to the storage type) and puts them into LDS in the
// convolution kernel's operand layout; the N x C weights of the 1x1 go there too.  After one barrier
// the waves (2 x 2 over pixels x output channels) run the C-deep product on the matrix cores and store
// through the convolution's epilogue (bias, residual, activation, one rounding).  The depthwise result
// never goes to memory and the 1x1 costs no launch of its own.
template <typename T, int C, int N, int BM>
__global__ __launch_bounds__(256) void dwconv_conv1x1_kernel(const DwArgs a, const ConvArgs c) {
    constexpr int CG = C / 8, PIECES = BM * CG / 256, WPIECES = N * CG / 256, TM = BM / 64, TN = N / 64;
    static_assert(256 % CG == 0 && PIECES >= 1 && PIECES <= 4 && WPIECES >= 1 && TM >= 1 && TN >= 1, "channel counts");
    typedef typename Mfma<T>::v8 v8;
    __shared__ __attribute__((aligned(16))) T sX[BM * C];
    __shared__ __attribute__((aligned(16))) T sW[N * C];
    const unsigned tid = threadIdx.x;
    const unsigned m0 = xcd_block(blockIdx.x, gridDim.x) * (unsigned)BM;
    const unsigned M = (unsigned)a.B * a.Ho * a.Wo;
    const int lane = tid & 63, wave = tid >> 6;
    const EpiPos pos{(int)m0, 0, (wave >> 1) * (BM / 2), (wave & 1) * (N / 2), lane & 31, lane >> 5};
    EpiOperands<TM, TN> eo;
    epilogue_load<TM, TN>(eo, c, pos);   // bias and residual of the 1x1, requested first
    uint4 wraw[WPIECES];
#pragma unroll
    for (int j = 0; j < WPIECES; ++j) {
        const unsigned cid = tid + j * 256u;
        wraw[j] = *reinterpret_cast<const uint4 *>(static_cast<const T *>(c.w) + (cid / CG) * C + (cid % CG) * 8u);
    }
    // this thread's channel group is the same for all its pieces: its nine filter taps and its bias once
    const unsigned cg = tid % CG;
    uint4 fw[9];
#pragma unroll
    for (int k = 0; k < 9; ++k) fw[k] = *reinterpret_cast<const uint4 *>(static_cast<const T *>(a.w) + k * C + cg * 8u);
    const float4 b0 = *reinterpret_cast<const float4 *>(a.bias + cg * 8u);
    const float4 b1 = *reinterpret_cast<const float4 *>(a.bias + cg * 8u + 4u);
    uint4 raw[PIECES][9];
    bool ok[PIECES][9];
#pragma unroll
    for (int j = 0; j < PIECES; ++j) {
        const unsigned m = min(m0 + (tid + j * 256u) / CG, M - 1u);   // rows beyond M: a valid pixel, never stored
        unsigned t = m / (unsigned)a.Wo;
        const int q = (int)(m - t * (unsigned)a.Wo);
        const unsigned n = t / (unsigned)a.Ho;
        const int p = (int)(t - n * (unsigned)a.Ho);
        const T *xg = static_cast<const T *>(a.x) + cg * 8u;
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s2 = 0; s2 < 3; ++s2) {
                const int ih = p * a.stride - a.pad + r, iw = q * a.stride - a.pad + s2;
                ok[j][r * 3 + s2] = (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
                const unsigned ihc = (unsigned)min(max(ih, 0), a.H - 1), iwc = (unsigned)min(max(iw, 0), a.W - 1);
                raw[j][r * 3 + s2] = *reinterpret_cast<const uint4 *>(xg + ((n * (unsigned)a.H + ihc) * (unsigned)a.W + iwc) * (unsigned)a.ldx);
            }
    }
#pragma unroll
    for (int j = 0; j < WPIECES; ++j) {
        const unsigned cid = tid + j * 256u;
        *reinterpret_cast<uint4 *>(sW + swz<C>((int)(cid / CG), (int)(cid % CG))) = wraw[j];
    }
#pragma unroll
    for (int j = 0; j < PIECES; ++j) {
        float acc[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
        for (int k = 0; k < 9; ++k) {
            const T *xe = reinterpret_cast<const T *>(&raw[j][k]);
            const T *we = reinterpret_cast<const T *>(&fw[k]);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = ok[j][k] ? acc[e] + (float)xe[e] * (float)we[e] : acc[e];
        }
        T out[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = (T)dw_act(acc[e], a.act);
        *reinterpret_cast<uint4 *>(sX + swz<C>((int)((tid + j * 256u) / CG), (int)cg)) = *reinterpret_cast<const uint4 *>(out);
    }
    __syncthreads();
    f32x16 accm[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) accm[i][j][e] = 0.f;
#pragma unroll
    for (int kk = 0; kk < C / 16; ++kk) {
        v8 fx[TM], fwv[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) fx[i] = *reinterpret_cast<const v8 *>(sX + swz<C>(pos.wm0 + i * 32 + pos.lrow, kk * 2 + pos.lhalf));
#pragma unroll
        for (int j = 0; j < TN; ++j) fwv[j] = *reinterpret_cast<const v8 *>(sW + swz<C>(pos.wn0 + j * 32 + pos.lrow, kk * 2 + pos.lhalf));
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) accm[i][j] = Mfma<T>::mma(fwv[j], fx[i], accm[i][j]);
    }
    epilogue_store<T, TM, TN>(accm, eo, c, pos);
}

// ---- a tensor into a channel range of a wider one (2-byte elements, 16 bytes per thread) ----
__global__ __launch_bounds__(256) void copy_channels_kernel(const CopyArgs a) {
    const unsigned c8 = (unsigned)a.C / 8u;
    const unsigned total = (unsigned)a.pixels * c8;
    const unsigned i = blockIdx.x * 256u + threadIdx.x;
    if (i >= total) return;
    const unsigned cg = i % c8, m = i / c8;
    const uint4 v = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(a.src) + (size_t)m * a.ld_src + cg * 8u);
    *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(a.dst) + (size_t)m * a.ld_dst + cg * 8u) = v;
}

// LOAD-time re-layout of depthwise weights: canonical W[C][1][kh][kw] -> [kh][kw][C].
__global__ __launch_bounds__(256) void pack_depthwise_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst, int C, int taps) {
    const size_t total = (size_t)C * taps;
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
        const int c = (int)(i % C), t = (int)(i / C);
        dst[i] = src[(size_t)c * taps + t];
    }
}

// ---- Winograd F(2x2, 3x3) transforms (3x3 stride-1 pad-1 convolution) ------------------------
//   Y = A^T [ (G g G^T) .* (B^T d B) ] A,  d = 4x4 input patch of a 2x2 output tile,
//   B^T = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1],  G = [1 0 0; .5 .5 .5; .5 -.5 .5; 0 0 1],
//   A^T = [1 1 1 0; 0 1 -1 -1].
// The element-wise product summed over input channels is 16 GEMMs [tiles x C] x [C x Cout], which
// run on the convolution kernel (batched 1x1 form).  The transforms are bandwidth-bound: one thread
// handles 8 channels of one tile, all accesses are 16-byte pieces contiguous across a wave.
template <typename T>
__global__ __launch_bounds__(256) void wino_input_kernel(const WinoArgs a) {
    const unsigned c8 = (unsigned)a.C / 8u;
    const unsigned tiles = (unsigned)a.B * a.th * a.tw;
    const unsigned i = blockIdx.x * 256u + threadIdx.x;
    if (i >= tiles * c8) return;
    const unsigned cg = i % c8, t = i / c8;
    const int tj = (int)(t % (unsigned)a.tw);
    const int ti = (int)((t / (unsigned)a.tw) % (unsigned)a.th);
    const unsigned n = t / ((unsigned)a.tw * a.th);
    const T *x = static_cast<const T *>(a.x);
    float d[4][4][8];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int ih = 2 * ti - 1 + r;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int iw = 2 * tj - 1 + s;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if ((unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W)
                v = *reinterpret_cast<const uint4 *>(x + ((size_t)(n * a.H + ih) * a.W + iw) * a.ldx + cg * 8u);
            const T *e = reinterpret_cast<const T *>(&v);
#pragma unroll
            for (int k = 0; k < 8; ++k) d[r][s][k] = (float)e[k];
        }
    }
    T *V = static_cast<T *>(a.y);
    const size_t plane = (size_t)tiles * a.C;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float u[4][4];   // B^T d
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            u[0][s] = d[0][s][k] - d[2][s][k];
            u[1][s] = d[1][s][k] + d[2][s][k];
            u[2][s] = d[2][s][k] - d[1][s][k];
            u[3][s] = d[1][s][k] - d[3][s][k];
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {   // (B^T d) B, back into d
            d[r][0][k] = u[r][0] - u[r][2];
            d[r][1][k] = u[r][1] + u[r][2];
            d[r][2][k] = u[r][2] - u[r][1];
            d[r][3][k] = u[r][1] - u[r][3];
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            T out[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) out[k] = (T)d[r][s][k];
            *reinterpret_cast<uint4 *>(V + (size_t)(r * 4 + s) * plane + (size_t)t * a.C + cg * 8u) = *reinterpret_cast<const uint4 *>(out);
        }
}

template <typename T>
__global__ __launch_bounds__(256) void wino_output_kernel(const WinoArgs a) {
    const unsigned c8 = (unsigned)a.C / 8u;
    const unsigned tiles = (unsigned)a.B * a.th * a.tw;
    const unsigned i = blockIdx.x * 256u + threadIdx.x;
    if (i >= tiles * c8) return;
    const unsigned cg = i % c8, t = i / c8;
    const int tj = (int)(t % (unsigned)a.tw);
    const int ti = (int)((t / (unsigned)a.tw) % (unsigned)a.th);
    const unsigned n = t / ((unsigned)a.tw * a.th);
    const T *M = static_cast<const T *>(a.x);
    const size_t plane = (size_t)tiles * a.C;
    float mm[4][4][8];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const uint4 v = *reinterpret_cast<const uint4 *>(M + (size_t)(r * 4 + s) * plane + (size_t)t * a.C + cg * 8u);
            const T *e = reinterpret_cast<const T *>(&v);
#pragma unroll
            for (int k = 0; k < 8; ++k) mm[r][s][k] = (float)e[k];
        }
    float bias[8];
    {
        const float4 b0 = *reinterpret_cast<const float4 *>(a.bias + cg * 8u);
        const float4 b1 = *reinterpret_cast<const float4 *>(a.bias + cg * 8u + 4u);
        bias[0] = b0.x; bias[1] = b0.y; bias[2] = b0.z; bias[3] = b0.w;
        bias[4] = b1.x; bias[5] = b1.y; bias[6] = b1.z; bias[7] = b1.w;
    }
    float y[2][2][8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float u[2][4];   // A^T m
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            u[0][s] = mm[0][s][k] + mm[1][s][k] + mm[2][s][k];
            u[1][s] = mm[1][s][k] - mm[2][s][k] - mm[3][s][k];
        }
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            y[r][0][k] = u[r][0] + u[r][1] + u[r][2] + bias[k];
            y[r][1][k] = u[r][1] - u[r][2] - u[r][3] + bias[k];
        }
    }
    T *Y = static_cast<T *>(a.y);
    const T *R = static_cast<const T *>(a.res);
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int oh = 2 * ti + r, ow = 2 * tj + s;
            if (oh >= a.H || ow >= a.W) continue;
            const size_t at = ((size_t)(n * a.H + oh) * a.W + ow) * a.C + cg * 8u;
            float v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = y[r][s][k];
            if (R) {
                const uint4 rv = *reinterpret_cast<const uint4 *>(R + at);
                const T *re = reinterpret_cast<const T *>(&rv);
#pragma unroll
                for (int k = 0; k < 8; ++k) v[k] += (float)re[k];
            }
            T out[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) out[k] = (T)dw_act(v[k], a.act);
            *reinterpret_cast<uint4 *>(Y + at) = *reinterpret_cast<const uint4 *>(out);
        }
}

// LOAD-time: W[cout][cin][3][3] -> U[16][cout'][cin], U = G g G^T in fp32, one rounding to T.
template <typename T>
__global__ __launch_bounds__(256) void pack_winograd_kernel(const T *__restrict__ src, T *__restrict__ dst, int cout, int cin) {
    const size_t total = (size_t)cout * cin;
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
        const int c = (int)(i % cin);
        const int kp = (int)(i / cin);   // row of the packed matrix
        const int row = kp & 31, g = row >> 3, h = (row >> 2) & 1, kk = row & 3;
        const int k = (kp & ~31) + (g >> 1) * 16 + h * 8 + (g & 1) * 4 + kk;   // the channel that row holds
        float w[3][3];
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s) w[r][s] = (float)src[(((size_t)k * cin + c) * 3 + r) * 3 + s];
        float gg[4][3];   // G g
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            gg[0][s] = w[0][s];
            gg[1][s] = 0.5f * (w[0][s] + w[1][s] + w[2][s]);
            gg[2][s] = 0.5f * (w[0][s] - w[1][s] + w[2][s]);
            gg[3][s] = w[2][s];
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float u0 = gg[r][0], u1 = 0.5f * (gg[r][0] + gg[r][1] + gg[r][2]), u2 = 0.5f * (gg[r][0] - gg[r][1] + gg[r][2]), u3 = gg[r][2];
            dst[(size_t)(r * 4 + 0) * total + i] = (T)u0;
            dst[(size_t)(r * 4 + 1) * total + i] = (T)u1;
            dst[(size_t)(r * 4 + 2) * total + i] = (T)u2;
            dst[(size_t)(r * 4 + 3) * total + i] = (T)u3;
        }
    }
}

// Workgroups of a LOAD-side launch: at most one per compute unit, each striding over its tensor.
// (Measured with EXECs running beside continuous LOADs: caps of 16, 48, 256 and no cap all leave
// the EXEC p50 within 0.6 % of EXEC alone; a LOAD of ResNet-50 takes 5.4, 2.6, 1.4 and 1.2 ms.)
constexpr unsigned kLoadGridCap = 256;

// row i of every group of 32 output channels receives channel sigma(i) of that group,
//     i = 8g + 4h + k  ->  sigma(i) = 16*(g/2) + 8h + 4*(g%2) + k,
// the order in which the conv kernel's MFMA accumulators come out as runs of 8 channels.
__global__ __launch_bounds__(256) void pack_weights_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst,
                                                           int cout, int cin, int kh, int kw, int khp, int kwp, int cinp,
                                                           int permute) {
    // A bounded grid that strides over the tensor: LOAD runs beside EXEC (paper section 5.2), and a
    // launch as wide as a large tensor would queue thousands of workgroups behind the EXEC kernels' own.
    const size_t total = (size_t)cout * khp * kwp * cinp;
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
        const int c = (int)(i % cinp);
        size_t t = i / cinp;
        const int s = (int)(t % kwp);
        t /= kwp;
        const int r = (int)(t % khp);
        int k = (int)(t / khp);
        if (permute) {
            const int row = k & 31, g = row >> 3, h = (row >> 2) & 1, kk = row & 3;
            k = (k & ~31) + (g >> 1) * 16 + h * 8 + (g & 1) * 4 + kk;
        }
        uint16_t v = 0;
        if (c < cin && s < kw && r < kh) v = src[(((size_t)k * cin + c) * kh + r) * kw + s];
        dst[i] = v;
    }
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
                                                               int B, int C, int H, int W, int ld) {
    const size_t total = (size_t)B * C * H * W;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;  // NCHW index
    if (i >= total) return;
    const int w = (int)(i % W);
    size_t t = i / W;
    const int h = (int)(t % H);
    t /= H;
    const int c = (int)(t % C);
    const int n = (int)(t / C);
    dst[i] = (float)src[(((size_t)n * H + h) * W + w) * ld + c];
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
    if (a.C < 1 || a.C > 4 || a.B < 1 || a.pad < 0 || a.Hp != a.H + 2 * a.pad || a.Wp < a.W + 2 * a.pad) return hipErrorInvalidValue;
    const size_t total = (size_t)a.B * a.Hp * a.Wp;
    if (total >= (1ull << 31)) return hipErrorInvalidValue;
    CW_DISPATCH(dt, cast_input_kernel, dim3(blocks_for(total, 256)), 256, s, a.x, a.y, a.B, a.C, a.H, a.W, a.pad, a.Hp, a.Wp);
    return hipGetLastError();
}

hipError_t launch_maxpool(DType dt, const PoolArgs &a, hipStream_t s) {
    if (a.C % 8 != 0 || a.B < 1) return hipErrorInvalidValue;
    const size_t total = (size_t)a.B * a.Ho * a.Wo * (a.C / 8);
    const bool small = total * 8 < (1ull << 31) && (size_t)a.H * a.W * a.C < (1ull << 31) && a.H > 0 && a.W > 0;
    if (a.k == 3 && small) {
        if (dt == DT_F16) maxpool_window_kernel<f16, 3><<<dim3(blocks_for(total, 256)), 256, 0, s>>>(a.x, a.y, a.B, a.H, a.W, a.C, a.Ho, a.Wo, a.k, a.stride, a.pad);
        else maxpool_window_kernel<bf16, 3><<<dim3(blocks_for(total, 256)), 256, 0, s>>>(a.x, a.y, a.B, a.H, a.W, a.C, a.Ho, a.Wo, a.k, a.stride, a.pad);
        return hipGetLastError();
    }
    CW_DISPATCH(dt, maxpool_kernel, dim3(blocks_for(total, 256)), 256, s, a);
    return hipGetLastError();
}

hipError_t launch_maxpool_conv(DType dt, const PoolArgs &a, const ConvArgs &c, int bm, hipStream_t s) {
    const size_t M = (size_t)a.B * a.Ho * a.Wo;
    if (a.C != 64 || a.k != 3 || a.B < 1 || M * 8 >= (1ull << 31) || (size_t)a.B * a.H * a.W * a.C >= (1ull << 31)) return hipErrorInvalidValue;
    if (c.Cin != 64 || c.K != 64 || (c.Cout != 64 && c.Cout != 128) || (size_t)c.M != M || c.res || !c.w || !c.bias || !c.y || !a.x || !a.y) return hipErrorInvalidValue;
    if (conv_ldy(c) < c.Cout || (bm != 64 && bm != 128)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((M + bm - 1) / bm));
#define CW_POOLCONV(BM_, N_)                                                                  \
    do {                                                                                      \
        if (dt == DT_F16) maxpool_conv1x1_kernel<f16, 3, BM_, N_><<<grid, 256, 0, s>>>(a, c); \
        else maxpool_conv1x1_kernel<bf16, 3, BM_, N_><<<grid, 256, 0, s>>>(a, c);             \
    } while (0)
    if (bm == 64 && c.Cout == 64) CW_POOLCONV(64, 64);
    else if (bm == 64) CW_POOLCONV(64, 128);
    else if (c.Cout == 64) CW_POOLCONV(128, 64);
    else CW_POOLCONV(128, 128);
#undef CW_POOLCONV
    return hipGetLastError();
}

// 128 channels have the kernel too, but there the 32 KB of weights that every 64-pixel workgroup fetches make the launch
// slower than the two it replaces (26.7 against 25.7 us over 50176 pixels): not planned.
bool dwconv_conv_ok(int c, int n) { return (c == 32 || c == 64) && (n == 64 || n == 128); }

int dwconv_conv_bm(int c, long long M) {
    // Measured on the MobileNet list: 128 or 256 pixels per workgroup (more window loads in flight per thread, the
    // 1x1's weights fetched by fewer workgroups) made the 32-channel launch slower (21.6 against 20.1 us over 200704
    // pixels) and the 64-channel one 1 us faster; 64 pixels everywhere.
    (void)c; (void)M;
    return 64;
}

hipError_t launch_dwconv_conv(DType dt, const DwArgs &a, const ConvArgs &c, hipStream_t s) {
    const size_t M = (size_t)a.B * a.Ho * a.Wo;
    if (!dwconv_conv_ok(a.C, c.Cout) || a.kh != 3 || a.kw != 3 || a.B < 1 || a.res || !a.x || !a.w || !a.bias || a.ldx < a.C) return hipErrorInvalidValue;
    if (M * 16 >= (1ull << 31) || (size_t)a.B * a.H * a.W * a.ldx >= (1ull << 31)) return hipErrorInvalidValue;
    if (c.Cin != a.C || c.K != a.C || (size_t)c.M != M || !c.w || !c.bias || !c.y || conv_ldy(c) < c.Cout) return hipErrorInvalidValue;
    const int bm = dwconv_conv_bm(a.C, (long long)M);
    const dim3 grid((unsigned)((M + bm - 1) / bm));
#define CW_DWPW(C_, N_, BM_)                                                                      \
    do {                                                                                          \
        if (dt == DT_F16) dwconv_conv1x1_kernel<f16, C_, N_, BM_><<<grid, 256, 0, s>>>(a, c);     \
        else dwconv_conv1x1_kernel<bf16, C_, N_, BM_><<<grid, 256, 0, s>>>(a, c);                 \
    } while (0)
#define CW_DWPW_N(C_, BM_)                          \
    do {                                            \
        if (c.Cout == 64) CW_DWPW(C_, 64, BM_);     \
        else CW_DWPW(C_, 128, BM_);                 \
    } while (0)
    if (bm != 64) return hipErrorInvalidValue;
    if (a.C == 32) CW_DWPW_N(32, 64);
    else CW_DWPW_N(64, 64);
#undef CW_DWPW_N
#undef CW_DWPW
    return hipGetLastError();
}

hipError_t launch_gavgpool(DType dt, const PoolArgs &a, hipStream_t s) {
    if (a.C % 8 != 0 || a.B < 1) return hipErrorInvalidValue;
    if (a.C % 64 != 0) return hipErrorInvalidValue;
    if (a.H * a.W >= kGapWideFrom)
        CW_DISPATCH(dt, gavgpool_wide_kernel, dim3((unsigned)(a.B * (a.C / 64))), 64 * kGapWaves, s, a.x, a.y, a.B, a.H, a.W, a.C, a.Ho, a.Wo, a.k, a.stride, a.pad);
    else
        CW_DISPATCH(dt, gavgpool_kernel, dim3((unsigned)(a.B * (a.C / 64))), 64, s, a.x, a.y, a.B, a.H, a.W, a.C, a.Ho, a.Wo, a.k, a.stride, a.pad);
    return hipGetLastError();
}

hipError_t launch_fc(DType dt, const FcArgs &a, hipStream_t s) {
    if (a.p) {   // FC + softmax in one launch
        const int S = a.split_k;
        if (a.B < 1 || a.B > kFcSoftmaxMaxBatch || a.Out < 1 || a.Out > kFcSoftmaxMaxOut || (S != 1 && S != 2 && S != 4) ||
            a.In % (32 * kFcsWaves * S) != 0 || !a.counters || (S > 1 && !a.partial))
            return hipErrorInvalidValue;
        CW_DISPATCH(dt, fc_softmax_kernel, dim3(blocks_for(a.Out, 16), S), 64 * kFcsWaves, s, a.f, a.w, a.bias, a.z, a.p, a.partial,
                    a.counters, a.B, a.In, a.Out, S);
        return hipGetLastError();
    }
    if (a.In % (32 * kFcWaves) != 0 || a.B < 1 || a.Out < 1) return hipErrorInvalidValue;
    const dim3 grid(blocks_for(a.Out, 16), blocks_for(a.B, 16));
    CW_DISPATCH(dt, fc_kernel, grid, 64 * kFcWaves, s, a.f, a.w, a.bias, a.z, a.B, a.In, a.Out);
    return hipGetLastError();
}

hipError_t launch_softmax(const SoftmaxArgs &a, hipStream_t s) {
    if (a.B < 1 || a.D < 1) return hipErrorInvalidValue;
    if (a.D <= 256 * 4)
        softmax_rows_kernel<4><<<dim3(a.B), 256, 0, s>>>(a.z, a.p, a.B, a.D);
    else if (a.D <= 256 * 16)
        softmax_rows_kernel<16><<<dim3(a.B), 256, 0, s>>>(a.z, a.p, a.B, a.D);
    else
        softmax_kernel<<<dim3(a.B), 256, 0, s>>>(a);
    return hipGetLastError();
}

hipError_t launch_pack_weights(const void *src, void *dst, int cout, int cin, int kh, int kw, int khp, int kwp, int cinp,
                               bool permute, hipStream_t s) {
    if (permute && cout % 32 != 0) return hipErrorInvalidValue;
    const size_t total = (size_t)cout * khp * kwp * cinp;
    const unsigned want = blocks_for(total, 256);
    pack_weights_kernel<<<dim3(want < kLoadGridCap ? want : kLoadGridCap), 256, 0, s>>>(static_cast<const uint16_t *>(src),
                                                                    static_cast<uint16_t *>(dst), cout, cin, kh, kw,
                                                                    khp, kwp, cinp, permute ? 1 : 0);
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

hipError_t launch_nhwc_to_nchw_f32(DType dt, const void *src, float *dst, int B, int C, int H, int W, int ld, hipStream_t s) {
    const size_t total = (size_t)B * C * H * W;
    if (ld < C) return hipErrorInvalidValue;
    if (dt == DT_F16)
        nhwc_to_nchw_f32_kernel<f16><<<dim3(blocks_for(total, 256)), 256, 0, s>>>(static_cast<const f16 *>(src), dst, B, C, H, W, ld);
    else
        nhwc_to_nchw_f32_kernel<bf16><<<dim3(blocks_for(total, 256)), 256, 0, s>>>(static_cast<const bf16 *>(src), dst, B, C, H, W, ld);
    return hipGetLastError();
}

hipError_t launch_dwconv(DType dt, const DwArgs &a, hipStream_t s) {
    // shapes the kernel's indexing relies on, checked here so that a bad launch is an error
    if (a.C < 8 || a.C % 8 != 0 || a.ldx < a.C || a.ldy < a.C || a.ldx % 8 != 0 || a.ldy % 8 != 0) return hipErrorInvalidValue;
    if (a.B < 1 || a.kh < 1 || a.kw < 1 || a.stride < 1 || a.pad < 0 || a.H < 1 || a.W < 1) return hipErrorInvalidValue;
    if (a.Ho != (a.H + 2 * a.pad - a.kh) / a.stride + 1 || a.Wo != (a.W + 2 * a.pad - a.kw) / a.stride + 1 || a.Ho < 1 || a.Wo < 1) return hipErrorInvalidValue;
    if (!a.x || !a.w || !a.bias || !a.y) return hipErrorInvalidValue;
    const size_t total = (size_t)a.B * a.Ho * a.Wo * (a.C / 8);
    if (total >= (1ull << 31) || (size_t)a.B * a.H * a.W * a.ldx >= (1ull << 31) || (size_t)a.B * a.Ho * a.Wo * a.ldy >= (1ull << 31)) return hipErrorInvalidValue;
    CW_DISPATCH(dt, dwconv_kernel, dim3(blocks_for(total, 256)), 256, s, a);
    return hipGetLastError();
}

hipError_t launch_copy_channels(const CopyArgs &a, hipStream_t s) {
    if (a.C < 8 || a.C % 8 != 0 || a.ld_src < a.C || a.ld_dst < a.C || a.ld_src % 8 != 0 || a.ld_dst % 8 != 0 || a.pixels < 1 || !a.src || !a.dst)
        return hipErrorInvalidValue;
    const size_t total = (size_t)a.pixels * (a.C / 8);
    if (total >= (1ull << 31)) return hipErrorInvalidValue;
    copy_channels_kernel<<<dim3(blocks_for(total, 256)), 256, 0, s>>>(a);
    return hipGetLastError();
}

static hipError_t wino_check(const WinoArgs &a, bool input) {
    if (a.B < 1 || a.H < 1 || a.W < 1 || a.C < 8 || a.C % 8 != 0 || !a.x || !a.y) return hipErrorInvalidValue;
    if (a.th != (a.H + 1) / 2 || a.tw != (a.W + 1) / 2) return hipErrorInvalidValue;
    if (input ? (a.ldx < a.C || a.ldx % 8 != 0) : !a.bias) return hipErrorInvalidValue;
    const size_t tiles = (size_t)a.B * a.th * a.tw;
    if (16 * tiles * a.C >= (1ull << 31) || (size_t)a.B * a.H * a.W * (input ? a.ldx : a.C) >= (1ull << 31)) return hipErrorInvalidValue;
    return hipSuccess;
}

hipError_t launch_wino_input(DType dt, const WinoArgs &a, hipStream_t s) {
    const hipError_t e = wino_check(a, true);
    if (e != hipSuccess) return e;
    const size_t total = (size_t)a.B * a.th * a.tw * (a.C / 8);
    CW_DISPATCH(dt, wino_input_kernel, dim3(blocks_for(total, 256)), 256, s, a);
    return hipGetLastError();
}

hipError_t launch_wino_output(DType dt, const WinoArgs &a, hipStream_t s) {
    const hipError_t e = wino_check(a, false);
    if (e != hipSuccess) return e;
    const size_t total = (size_t)a.B * a.th * a.tw * (a.C / 8);
    CW_DISPATCH(dt, wino_output_kernel, dim3(blocks_for(total, 256)), 256, s, a);
    return hipGetLastError();
}

hipError_t launch_pack_winograd(DType dt, const void *src, void *dst, int cout, int cin, hipStream_t s) {
    if (cout < 32 || cout % 32 != 0 || cin < 1) return hipErrorInvalidValue;
    const unsigned want = blocks_for((size_t)cout * cin, 256);
    const dim3 grid(want < kLoadGridCap ? want : kLoadGridCap);
    if (dt == DT_F16) pack_winograd_kernel<f16><<<grid, 256, 0, s>>>(static_cast<const f16 *>(src), static_cast<f16 *>(dst), cout, cin);
    else pack_winograd_kernel<bf16><<<grid, 256, 0, s>>>(static_cast<const bf16 *>(src), static_cast<bf16 *>(dst), cout, cin);
    return hipGetLastError();
}

hipError_t launch_pack_depthwise(const void *src, void *dst, int c, int kh, int kw, hipStream_t s) {
    if (c < 1 || kh < 1 || kw < 1) return hipErrorInvalidValue;
    const unsigned want = blocks_for((size_t)c * kh * kw, 256);
    pack_depthwise_kernel<<<dim3(want < kLoadGridCap ? want : kLoadGridCap), 256, 0, s>>>(static_cast<const uint16_t *>(src), static_cast<uint16_t *>(dst), c, kh * kw);
    return hipGetLastError();
}

}  // namespace cw
