// Shared pieces of the convolution kernels: MFMA wrappers, buffer descriptors, the LDS swizzle
// and the fused epilogue (bias + residual + ReLU + store, and the in-kernel split-K reduction).
#pragma once
#include "common.h"

namespace cw {
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr unsigned kOob = 0x80000000u;  // byte offset beyond any buffer (buffers are < 2 GiB)

enum ConvMode : int { MODE_CONV = 0, MODE_GEMM = 1, MODE_STEM = 2 };

// n / d for a divisor prepared on the host (round-up multiplier; exact for every 32-bit n).
static __device__ __forceinline__ unsigned fast_div(unsigned n, const FastDiv &d) {
    const unsigned t = __umulhi(d.magic, n);
    return (t + ((n - t) >> d.sh1)) >> d.sh2;
}

static __device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, unsigned bytes) {
    // raw buffer (stride 0), 32-bit data format word as on every CDNA part
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, bytes, 0x00020000);
}

template <typename T>
struct Mfma;
template <>
struct Mfma<f16> {
    typedef _Float16 v8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ f32x16 mma(v8 rows, v8 cols, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(rows, cols, c, 0, 0, 0);
    }
};
template <>
struct Mfma<bf16> {
    typedef __bf16 v8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ f32x16 mma(v8 rows, v8 cols, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(rows, cols, c, 0, 0, 0);
    }
};

// Element offset of 16-byte chunk c of `row` inside a [rows][BK] LDS stage.  A 16-byte-per-lane
// LDS access is served 16 lanes (256 bytes, all 64 banks) per clock, and an MFMA operand read
// has 16 consecutive rows at one chunk index in such a group.  With 128-byte rows two rows
// share 256 bytes, so the chunk index is XORed with (row/2)%8: rows of equal parity then land
// on 8 different chunk positions and the two parities on the two halves.  With 64-byte rows
// four rows share 256 bytes and the key is (row/4)%4; with 256-byte rows every row covers all
// banks and the key is row%16.
template <int BK>
static __device__ __forceinline__ int swz_key(int row) {
    return BK == 128 ? (row & 15) : BK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}
template <int BK>
static __device__ __forceinline__ int swz(int row, int c) {
    return row * BK + ((c ^ swz_key<BK>(row)) << 3);
}

// ---- epilogue ------------------------------------------------------------------------------
// Accumulator layout (weights are the MFMA row operand, pixels the column operand): the lane
// holds pixel m0+wm0+32i+lane%32; of channel tile j its registers 8q..8q+7 are channels
// n0+wn0+32j+16q+8*(lane/32) .. +7  (q = 0, 1).
struct EpiPos {
    int m0, n0, wm0, wn0, lrow, lhalf;
};

// Split-K: every workgroup of a tile stores its raw fp32 partial tile, then takes a ticket.
// The one that draws the last ticket adds the partial tiles of all splits in split order (its
// own included, re-read like the others, so the sum does not depend on which workgroup came
// last) and returns true; the others return false and are done.
// Workgroups of one tile may sit on different XCDs, whose L2s are not coherent for plain
// accesses.  The partial sums therefore travel as device-scope accesses (sc1: stores write
// through, loads do not hit a stale local line), which costs no cache-wide write-back or
// invalidate; a store is complete once vmcnt has counted it.
template <int TM, int TN>
static __device__ __forceinline__ bool splitk_exchange(f32x16 (&acc)[TM][TN], const ConvArgs &a, const EpiPos &p, int tile_id) {
    constexpr int kDeviceScope = 16;  // cache-policy operand: sc1
    __shared__ int s_last;
    const unsigned mn = (unsigned)a.M * a.Cout;
    {
        const __amdgpu_buffer_rsrc_t rp = make_rsrc(a.partial + (size_t)blockIdx.y * a.M * a.Cout, mn * 4u);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const unsigned m = p.m0 + p.wm0 + i * 32 + p.lrow;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const unsigned n = p.n0 + p.wn0 + j * 32 + q * 16 + p.lhalf * 8;
                    const unsigned o = (m < (unsigned)a.M && n < (unsigned)a.Cout) ? (m * a.Cout + n) * 4u : kOob;
                    const f32x16 &v = acc[i][j];
                    __builtin_amdgcn_raw_buffer_store_b128(
                        u32x4{__float_as_uint(v[8 * q + 0]), __float_as_uint(v[8 * q + 1]), __float_as_uint(v[8 * q + 2]),
                              __float_as_uint(v[8 * q + 3])},
                        rp, o, 0, kDeviceScope);
                    __builtin_amdgcn_raw_buffer_store_b128(
                        u32x4{__float_as_uint(v[8 * q + 4]), __float_as_uint(v[8 * q + 5]), __float_as_uint(v[8 * q + 6]),
                              __float_as_uint(v[8 * q + 7])},
                        rp, o + 16u, 0, kDeviceScope);
                }
        }
    }
    __builtin_amdgcn_s_waitcnt(0);  // vmcnt(0): this thread's partial sums have been written
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();  // ... and so have those of the whole workgroup
    if (threadIdx.x == 0) {
        const int ticket = __hip_atomic_fetch_add(&a.counters[tile_id], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = ticket == a.split_k - 1;
        if (last) __hip_atomic_store(&a.counters[tile_id], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next launch
        s_last = last;
    }
    __syncthreads();
    if (!s_last) return false;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    for (int z = 0; z < a.split_k; ++z) {
        const __amdgpu_buffer_rsrc_t rp = make_rsrc(a.partial + (size_t)z * a.M * a.Cout, mn * 4u);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const unsigned m = p.m0 + p.wm0 + i * 32 + p.lrow;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const unsigned n = p.n0 + p.wn0 + j * 32 + q * 16 + p.lhalf * 8;
                    const unsigned o = (m < (unsigned)a.M && n < (unsigned)a.Cout) ? (m * a.Cout + n) * 4u : kOob;
                    const u32x4 p0 = __builtin_amdgcn_raw_buffer_load_b128(rp, o, 0, kDeviceScope);
                    const u32x4 p1 = __builtin_amdgcn_raw_buffer_load_b128(rp, o + 16u, 0, kDeviceScope);
                    acc[i][j][8 * q + 0] += __uint_as_float(p0.x);
                    acc[i][j][8 * q + 1] += __uint_as_float(p0.y);
                    acc[i][j][8 * q + 2] += __uint_as_float(p0.z);
                    acc[i][j][8 * q + 3] += __uint_as_float(p0.w);
                    acc[i][j][8 * q + 4] += __uint_as_float(p1.x);
                    acc[i][j][8 * q + 5] += __uint_as_float(p1.y);
                    acc[i][j][8 * q + 6] += __uint_as_float(p1.z);
                    acc[i][j][8 * q + 7] += __uint_as_float(p1.w);
                }
        }
    }
    return true;
}

// Bias and residual operands of the epilogue, as 16-byte vectors.  Loading them is separate
// from using them so that a kernel can issue the loads before its last MFMAs.
template <int TM, int TN>
struct EpiOperands {
    u32x4 bv[TN][2][2], rv[TM][TN][2];
};

template <int TM, int TN>
static __device__ __forceinline__ void epilogue_load(EpiOperands<TM, TN> &e, const ConvArgs &a, const EpiPos &p) {
    const unsigned mn = (unsigned)a.M * a.Cout;
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(a.res ? a.res : a.y, mn * 2u);
    // without a bias (the batched form) every bias load is out of range and returns zeros
    const bool has_bias = a.bias != nullptr;
    const __amdgpu_buffer_rsrc_t rb = make_rsrc(has_bias ? static_cast<const void *>(a.bias) : a.y, (unsigned)a.Cout * 4u);
    const bool has_res = a.res != nullptr;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const unsigned n = p.n0 + p.wn0 + j * 32 + q * 16 + p.lhalf * 8;
            const unsigned o = (has_bias && n < (unsigned)a.Cout) ? n * 4u : kOob;
            e.bv[j][q][0] = __builtin_amdgcn_raw_buffer_load_b128(rb, o, 0, 0);
            e.bv[j][q][1] = __builtin_amdgcn_raw_buffer_load_b128(rb, has_bias ? o + 16u : kOob, 0, 0);
        }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const unsigned m = p.m0 + p.wm0 + i * 32 + p.lrow;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const unsigned n = p.n0 + p.wn0 + j * 32 + q * 16 + p.lhalf * 8;
                const unsigned o = (has_res && m < (unsigned)a.M && n < (unsigned)a.Cout) ? (m * a.Cout + n) * 2u : kOob;
                e.rv[i][j][q] = __builtin_amdgcn_raw_buffer_load_b128(rr, o, 0, 0);  // zeros without a residual
            }
    }
}

// + bias, + residual, activation, one round-to-nearest-even to the storage type, 16-byte stores.
// The activation code is uniform, so the hard-swish arithmetic sits behind a scalar branch and the
// ReLU / identity form runs the instructions it always ran.
template <typename T, int TM, int TN, bool HSWISH>
static __device__ __forceinline__ void epilogue_store_act(const f32x16 (&acc)[TM][TN], const EpiOperands<TM, TN> &e, const ConvArgs &a,
                                                          const EpiPos &p) {
    // y may be a channel range of a wider tensor: ldy elements from one pixel to the next
    const unsigned ldy = (unsigned)conv_ldy(a);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, (((unsigned)a.M - 1u) * ldy + (unsigned)a.Cout) * 2u);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const unsigned m = p.m0 + p.wm0 + i * 32 + p.lrow;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const unsigned n = p.n0 + p.wn0 + j * 32 + q * 16 + p.lhalf * 8;
                const unsigned o = (m < (unsigned)a.M && n < (unsigned)a.Cout) ? (m * ldy + n) * 2u : kOob;
                const T *r = reinterpret_cast<const T *>(&e.rv[i][j][q]);
                const float *b = reinterpret_cast<const float *>(&e.bv[j][q][0]);
                T out[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float v = acc[i][j][8 * q + k] + b[k] + (float)r[k];
                    if (HSWISH) out[k] = (T)(v * fminf(fmaxf(v + 3.f, 0.f), 6.f) * (1.f / 6.f));
                    else out[k] = (T)(a.relu ? fmaxf(v, 0.f) : v);
                }
                __builtin_amdgcn_raw_buffer_store_b128(*reinterpret_cast<const u32x4 *>(out), ry, o, 0, 0);
            }
    }
}

template <typename T, int TM, int TN>
static __device__ __forceinline__ void epilogue_store(const f32x16 (&acc)[TM][TN], const EpiOperands<TM, TN> &e, const ConvArgs &a,
                                                      const EpiPos &p) {
    if (a.relu == ACT_HSWISH) epilogue_store_act<T, TM, TN, true>(acc, e, a, p);
    else epilogue_store_act<T, TM, TN, false>(acc, e, a, p);
}

// Workgroups go to the 8 XCDs round-robin; give each XCD a contiguous run of tiles so that
// tiles sharing pixels (same tile_m) meet in one XCD's L2.
static __device__ __forceinline__ int xcd_tile_id(int bid, int nb) {
    const int xcd = bid & 7, idx = bid >> 3;
    const int per = nb >> 3, rem = nb & 7;
    return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}
static __device__ __forceinline__ int xcd_tile_id() { return xcd_tile_id(blockIdx.x, gridDim.x); }

}  // namespace cw
