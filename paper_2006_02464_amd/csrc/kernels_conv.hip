// Implicit-GEMM convolution on gfx950 MFMA (v_mfma_f32_32x32x16_{f16,bf16}), fp32 accumulate.
//
// GEMM view: M = B*Ho*Wo output pixels (rows, NHWC so a row of y is Cout contiguous values),
// N = Cout, K = kh*kwp*Cin ordered (r, s, c) so that for one filter tap the K slice is the
// Cin-contiguous run of one input pixel.  A (activations) is gathered on the fly with zero
// fill for padded taps; B (weights) was re-laid out at LOAD as [Cout][K].
//
// Per workgroup: a BM x BN output tile; K is walked in slices of 32 through two LDS stages
// (global -> registers -> LDS, one barrier per slice).  Each wave owns a (BM/WARPS_M) x
// (BN/WARPS_N) sub-tile made of 32x32 MFMA tiles.
//
// Epilogue (fused): + bias, + residual, ReLU, one round-to-nearest-even to the storage type.
// With split-K (gridDim.y > 1) the raw fp32 partial sums go to a [split][M][Cout] buffer and
// a second kernel reduces them in fixed order and applies the same epilogue.
#include "common.h"

namespace cw {

typedef float f32x16 __attribute__((ext_vector_type(16)));

template <typename T>
struct Mfma;
template <>
struct Mfma<f16> {
    typedef _Float16 v8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ f32x16 mma(v8 a, v8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};
template <>
struct Mfma<bf16> {
    typedef __bf16 v8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ f32x16 mma(v8 a, v8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};

constexpr int BK = 32;   // K slice per LDS stage
constexpr int BKP = 40;  // LDS row pitch in elements (80 B): conflict-free ds_read_b128

template <typename T, int BM, int BN, int WARPS_M, int WARPS_N, bool STEM>
__global__ __launch_bounds__(64 * WARPS_M * WARPS_N) void conv_igemm_kernel(const ConvArgs a) {
    constexpr int NT = 64 * WARPS_M * WARPS_N;
    constexpr int WM = BM / WARPS_M, WN = BN / WARPS_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_CHUNKS = BM * (BK / 8), B_CHUNKS = BN * (BK / 8);  // 16-byte chunks
    static_assert(A_CHUNKS % NT == 0 && B_CHUNKS % NT == 0, "tile/threads mismatch");
    constexpr int A_PER = A_CHUNKS / NT, B_PER = B_CHUNKS / NT;
    typedef typename Mfma<T>::v8 v8;

    __shared__ __attribute__((aligned(16))) T sA[2][BM * BKP];
    __shared__ __attribute__((aligned(16))) T sB[2][BN * BKP];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm0 = (wave / WARPS_N) * WM;
    const int wn0 = (wave % WARPS_N) * WN;

    const int tiles_n = (a.Cout + BN - 1) / BN;
    const int tile_m = blockIdx.x / tiles_n;
    const int tile_n = blockIdx.x - tile_m * tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int ktiles = a.K / BK;
    const int kt0 = blockIdx.y * a.ktiles_per_split;
    const int kt1 = min(ktiles, kt0 + a.ktiles_per_split);

    const T *__restrict__ xg = static_cast<const T *>(a.x);
    const T *__restrict__ wg = static_cast<const T *>(a.w);

    // Per-thread gather coordinates of its A chunks (fixed for the whole K walk).
    int a_pix[A_PER];  // element offset of x[n][0][0][0], or -1 if the row is beyond M
    int a_ih0[A_PER], a_iw0[A_PER];
#pragma unroll
    for (int j = 0; j < A_PER; ++j) {
        const int cid = tid + j * NT;
        const int m = m0 + (cid >> 2);
        if (m < a.M) {
            const int q = m % a.Wo;
            const int t = m / a.Wo;
            const int p = t % a.Ho;
            const int n = t / a.Ho;
            a_pix[j] = n * a.H * a.W * a.Cin;
            a_ih0[j] = p * a.stride - a.pad;
            a_iw0[j] = q * a.stride - a.pad;
        } else {
            a_pix[j] = -1;
            a_ih0[j] = 0;
            a_iw0[j] = 0;
        }
    }

    uint4 ra[A_PER], rb[B_PER];

    // (r, s, c0) of K slice kt: k0 = kt*32 = ((r*kwp + s)*Cin + c0).
    int fr, fs, fc0;
    if (STEM) {
        fr = kt0; fs = 0; fc0 = 0;
    } else {
        const int k0 = kt0 * BK;
        const int rs = k0 / a.Cin;
        fc0 = k0 - rs * a.Cin;
        fr = rs / a.kwp;
        fs = rs - fr * a.kwp;
    }

    auto load_global = [&](int kt) {
#pragma unroll
        for (int j = 0; j < A_PER; ++j) {
            const int cid = tid + j * NT;
            const int kc = cid & 3;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (STEM) {
                // Cin == 4, kwp == 8: slice kt is filter row r = kt; chunk kc holds taps 2kc, 2kc+1.
                const int ih = a_ih0[j] + fr;
                if (a_pix[j] >= 0 && (unsigned)ih < (unsigned)a.H) {
                    const int iw = a_iw0[j] + 2 * kc;
                    const T *row = xg + a_pix[j] + (ih * a.W) * 4;
                    if ((unsigned)iw < (unsigned)a.W) {
                        const uint2 t = *reinterpret_cast<const uint2 *>(row + iw * 4);
                        v.x = t.x; v.y = t.y;
                    }
                    if ((unsigned)(iw + 1) < (unsigned)a.W) {
                        const uint2 t = *reinterpret_cast<const uint2 *>(row + (iw + 1) * 4);
                        v.z = t.x; v.w = t.y;
                    }
                }
            } else {
                const int ih = a_ih0[j] + fr, iw = a_iw0[j] + fs;
                if (a_pix[j] >= 0 && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W)
                    v = *reinterpret_cast<const uint4 *>(xg + a_pix[j] + (ih * a.W + iw) * a.Cin + fc0 + kc * 8);
            }
            ra[j] = v;
        }
#pragma unroll
        for (int j = 0; j < B_PER; ++j) {
            const int cid = tid + j * NT;
            const int n = n0 + (cid >> 2);
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (n < a.Cout)
                v = *reinterpret_cast<const uint4 *>(wg + (size_t)n * a.K + kt * BK + (cid & 3) * 8);
            rb[j] = v;
        }
        // advance (r, s, c0) to the next slice
        if (STEM) {
            fr += 1;
        } else {
            fc0 += BK;
            if (fc0 == a.Cin) {
                fc0 = 0;
                if (++fs == a.kwp) { fs = 0; ++fr; }
            }
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int j = 0; j < A_PER; ++j) {
            const int cid = tid + j * NT;
            *reinterpret_cast<uint4 *>(&sA[buf][(cid >> 2) * BKP + (cid & 3) * 8]) = ra[j];
        }
#pragma unroll
        for (int j = 0; j < B_PER; ++j) {
            const int cid = tid + j * NT;
            *reinterpret_cast<uint4 *>(&sB[buf][(cid >> 2) * BKP + (cid & 3) * 8]) = rb[j];
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    if (kt0 < kt1) {
        load_global(kt0);
        store_lds(0);
    }
    __syncthreads();

    const int lrow = lane & 31;
    const int lk = (lane >> 5) * 8;
    for (int kt = kt0; kt < kt1; ++kt) {
        const int cur = (kt - kt0) & 1;
        const bool more = kt + 1 < kt1;
        if (more) load_global(kt + 1);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            v8 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const v8 *>(&sA[cur][(wm0 + i * 32 + lrow) * BKP + kk * 16 + lk]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const v8 *>(&sB[cur][(wn0 + j * 32 + lrow) * BKP + kk * 16 + lk]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = Mfma<T>::mma(fa[i], fb[j], acc[i][j]);
        }
        if (more) store_lds(cur ^ 1);
        __syncthreads();
    }

    // Epilogue.  Lane holds column n = lane%32 and rows 8*(e/4) + 4*(lane/32) + e%4 of each tile.
    const int rhalf = (lane >> 5) * 4;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn0 + j * 32 + lrow;
        if (n >= a.Cout) continue;
        const float bias = a.partial ? 0.f : a.bias[n];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm0 + i * 32 + 8 * (e >> 2) + rhalf + (e & 3);
                if (m >= a.M) continue;
                const size_t o = (size_t)m * a.Cout + n;
                if (a.partial) {
                    a.partial[(size_t)blockIdx.y * a.M * a.Cout + o] = acc[i][j][e];
                } else {
                    float v = acc[i][j][e] + bias;
                    if (a.res) v += (float)static_cast<const T *>(a.res)[o];
                    if (a.relu) v = fmaxf(v, 0.f);
                    static_cast<T *>(a.y)[o] = (T)v;
                }
            }
        }
    }
}

// Fixed-order reduction of split-K partials + the fused epilogue. One thread = 4 columns.
template <typename T>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const ReduceArgs a) {
    const size_t total4 = (size_t)a.M * a.Cout / 4;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total4) return;
    const size_t o = idx * 4;
    const int n = (int)(o % a.Cout);
    float4 s = *reinterpret_cast<const float4 *>(a.partial + o);
    for (int z = 1; z < a.split_k; ++z) {
        const float4 t = *reinterpret_cast<const float4 *>(a.partial + (size_t)z * a.M * a.Cout + o);
        s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    const float4 b = *reinterpret_cast<const float4 *>(a.bias + n);
    float v[4] = {s.x + b.x, s.y + b.y, s.z + b.z, s.w + b.w};
    if (a.res) {
        const T *r = static_cast<const T *>(a.res) + o;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] += (float)r[i];
    }
    T out[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) out[i] = (T)(a.relu ? fmaxf(v[i], 0.f) : v[i]);
    *reinterpret_cast<uint2 *>(static_cast<T *>(a.y) + o) = *reinterpret_cast<const uint2 *>(out);
}

TileDim conv_tile_dim(ConvTile t) {
    switch (t) {
        case T128x128: return {128, 128, 256};
        case T128x64: return {128, 64, 256};
        case T64x64: return {64, 64, 256};
        case T64x32: return {64, 32, 128};
        case T32x64: return {32, 64, 128};
        default: return {32, 32, 64};
    }
}

void conv_grid(ConvTile tile, const ConvArgs &a, dim3 *grid, int *block) {
    const TileDim d = conv_tile_dim(tile);
    const unsigned tm = (a.M + d.bm - 1) / d.bm, tn = (a.Cout + d.bn - 1) / d.bn;
    *grid = dim3(tm * tn, a.split_k, 1);
    *block = d.threads;
}

void reduce_grid(const ReduceArgs &a, dim3 *grid, int *block) {
    const size_t total4 = (size_t)a.M * a.Cout / 4;
    *grid = dim3((unsigned)((total4 + 255) / 256), 1, 1);
    *block = 256;
}

template <typename T, bool STEM>
static hipError_t launch_conv_t(ConvTile tile, const ConvArgs &a, hipStream_t s) {
    dim3 grid;
    int block;
    conv_grid(tile, a, &grid, &block);
    switch (tile) {
        case T128x128: conv_igemm_kernel<T, 128, 128, 2, 2, STEM><<<grid, block, 0, s>>>(a); break;
        case T128x64: conv_igemm_kernel<T, 128, 64, 2, 2, STEM><<<grid, block, 0, s>>>(a); break;
        case T64x64: conv_igemm_kernel<T, 64, 64, 2, 2, STEM><<<grid, block, 0, s>>>(a); break;
        case T64x32: conv_igemm_kernel<T, 64, 32, 2, 1, STEM><<<grid, block, 0, s>>>(a); break;
        case T32x64: conv_igemm_kernel<T, 32, 64, 1, 2, STEM><<<grid, block, 0, s>>>(a); break;
        case T32x32: conv_igemm_kernel<T, 32, 32, 1, 1, STEM><<<grid, block, 0, s>>>(a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_conv(DType dt, ConvTile tile, bool stem, const ConvArgs &a, hipStream_t s) {
    // Shapes the kernel's indexing relies on; the plan compiler guarantees them, checked again
    // here so that a bad launch is an error instead of an out-of-bounds access.
    if (a.K % BK != 0 || a.M <= 0 || a.Cout <= 0 || a.split_k < 1 || a.ktiles_per_split < 1)
        return hipErrorInvalidValue;
    if (stem ? (a.Cin != 4 || a.kwp != 8 || a.K != a.kh * 32) : (a.Cin % BK != 0 || a.kwp != a.kw))
        return hipErrorInvalidValue;
    if ((long long)a.split_k * a.ktiles_per_split < a.K / BK) return hipErrorInvalidValue;
    if (a.split_k > 1 && !a.partial) return hipErrorInvalidValue;
    if (dt == DT_F16)
        return stem ? launch_conv_t<f16, true>(tile, a, s) : launch_conv_t<f16, false>(tile, a, s);
    return stem ? launch_conv_t<bf16, true>(tile, a, s) : launch_conv_t<bf16, false>(tile, a, s);
}

hipError_t launch_splitk_reduce(DType dt, const ReduceArgs &a, hipStream_t s) {
    if (a.Cout % 4 != 0 || a.split_k < 1) return hipErrorInvalidValue;
    dim3 grid;
    int block;
    reduce_grid(a, &grid, &block);
    if (dt == DT_F16)
        splitk_reduce_kernel<f16><<<grid, block, 0, s>>>(a);
    else
        splitk_reduce_kernel<bf16><<<grid, block, 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace cw
