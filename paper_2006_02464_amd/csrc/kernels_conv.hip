// Implicit-GEMM convolution on gfx950 MFMA (v_mfma_f32_32x32x16_{f16,bf16}), fp32 accumulate:
// the register-staged kernel, the tile table and the launch entry point.
//
// launch_conv() sends every convolution with Cin % 64 == 0, and a first convolution with an even
// stride, to the direct-to-LDS kernel (kernels_conv_dlds.hip).  The kernel in this file serves
// what is left: Cin % 64 != 0 (K slices of 32) and a first convolution with an odd stride.  What
// follows describes the layout and conventions both kernels share, and this kernel's pipeline.
//
// GEMM view: M = B*Ho*Wo output pixels (NHWC, so a pixel's Cout values are contiguous),
// N = Cout, K = kh*kwp*Cin ordered (r, s, c), so that for one filter tap the K slice is the
// Cin-contiguous run of one input pixel.  Activations are gathered on the fly with zero fill
// for padded taps; weights were re-laid out at LOAD as [Cout'][K] (see "weight rows" below).
//
// Per workgroup: a BM-pixel x BN-channel output tile.  K is walked in slices of BK (64; 32 for
// the stem and for Cin % 64 != 0).  Slices travel global -> registers -> LDS: PF register sets
// hold the next PF slices in flight while the MFMAs consume the current one out of one of two
// LDS stages (one barrier per slice).  All global reads are raw buffer loads: a padded tap, a
// pixel beyond M or a slice beyond the K range gets a per-thread offset outside the buffer, for
// which the hardware returns zeros.  That keeps the steady-state loop free of branches, so the
// compiler waits for exactly the oldest register set (s_waitcnt vmcnt(n)) instead of draining
// every load in flight.  The per-thread part of an address is fixed for the whole K walk; the
// tap/channel part is uniform and rides in the instruction's scalar offset.
//
// LDS rows are BK elements with the 16-byte chunk index XOR-swizzled by the row, so both the
// 16-byte writes and the MFMA operand reads (lane = row, 8 consecutive k) are conflict free
// without padding (measured: 237 B/clk/CU for this read pattern against 123 with a key of
// row%8 and 31 without a swizzle).
//
// MFMA roles: the weight tile is the row operand, the pixel tile the column operand, so a lane
// ends up with 16 channels of ONE pixel per 32x32 tile.  Weight rows: inside every group of 32
// output channels the packer stores channel sigma(i) at row i, with
//     i = 8g + 4h + k  ->  sigma(i) = 16*(g/2) + 8h + 4*(g%2) + k,
// which makes those 16 accumulators two runs of 8 consecutive channels (registers 0..7 ->
// channels 8h..8h+7, registers 8..15 -> 16+8h..16+8h+7; h = lane/32).  The fused epilogue
// therefore works straight from registers: bias and residual arrive as 16-byte vectors, then
// + bias, + residual, ReLU, one round-to-nearest-even to the storage type, 16-byte stores;
// lanes l and l+32 complete 32 contiguous bytes of a pixel per store instruction.
// With split-K (gridDim.y > 1) the raw fp32 partial sums go to a [split][M][Cout] buffer; the
// workgroup of a tile that finishes last (an arrival counter per tile) adds them up in split
// order and applies the same epilogue, so no second launch is needed and the result does not
// depend on the order of arrival.
#include "conv_common.h"

namespace cw {

template <typename T, int BM, int BN, int WARPS_M, int WARPS_N, int BK, int PF, int MODE, bool SPLITK>
__global__ __launch_bounds__(64 * WARPS_M * WARPS_N) void conv_igemm_kernel(const ConvArgs a) {
    constexpr int NT = 64 * WARPS_M * WARPS_N;
    constexpr int WM = BM / WARPS_M, WN = BN / WARPS_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int CPR = BK / 8;  // 16-byte chunks per LDS row
    constexpr int X_CHUNKS = BM * CPR, W_CHUNKS = BN * CPR;
    static_assert(X_CHUNKS % NT == 0 && W_CHUNKS % NT == 0, "tile/threads mismatch");
    static_assert(MODE != MODE_STEM || BK == 32, "the stem walks one filter row (8 taps x 4 channels) per slice");
    constexpr int X_PER = X_CHUNKS / NT, W_PER = W_CHUNKS / NT;
    constexpr int STAGE = (BM + BN) * BK;  // elements per LDS stage
    typedef typename Mfma<T>::v8 v8;

    __shared__ __attribute__((aligned(16))) T lds[2 * STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm0 = (wave / WARPS_N) * WM;
    const int wn0 = (wave % WARPS_N) * WN;
    const int lrow = lane & 31;
    const int lhalf = lane >> 5;

    const int tile_id = xcd_tile_id();
    const int tiles_n = a.Cout / BN + (a.Cout % BN != 0);
    const int tile_m = tile_id / tiles_n;
    const int tile_n = tile_id - tile_m * tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int ktiles = a.K / BK;
    const int kt0 = blockIdx.y * a.ktiles_per_split;
    const int kt1 = min(ktiles, kt0 + a.ktiles_per_split);

    // The activation buffer is described from D bytes before its start, D = the offset of the
    // top-left tap relative to a filter's centre pixel, so that  centre offset (per thread, in a
    // VGPR) + tap/channel offset (uniform, in an SGPR)  is never negative.
    // x may be the first Cin channels of a wider tensor: ldx elements from one pixel to the next.
    const unsigned ldx = (unsigned)conv_ldx(a);
    const int pad_h = conv_pad_h(a), pad_w = conv_pad_w(a);
    const unsigned x_bytes = (((unsigned)a.B * a.H * a.W - 1u) * ldx + (unsigned)a.Cin) * 2u;
    const unsigned x_shift = MODE == MODE_GEMM ? 0u : (unsigned)(pad_h * a.W + pad_w) * ldx * 2u;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(static_cast<const char *>(a.x) - x_shift, x_bytes + x_shift);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(a.w, (unsigned)a.Cout * a.K * 2u);

    // Per-thread gather state of its activation chunks, fixed for the whole K walk: byte offset
    // of the chunk at the filter's centre pixel, and which taps fall inside the image.
    //   conv: bit r*kw+s of x_mask = tap (r, s) is in range (kh*kw <= 32);
    //   gemm: bit 0 = the pixel exists (1x1, stride 1, no padding: x is a plain [M][Cin] matrix);
    //   stem: bits 0..kh-1 = filter row r is in range, bits 30/31 = the chunk's two columns are.
    unsigned x_voff[X_PER], x_mask[X_PER];
#pragma unroll
    for (int j = 0; j < X_PER; ++j) {
        const int cid = tid + j * NT;
        const int c = cid % CPR;
        const unsigned m = m0 + cid / CPR;
        unsigned mask = 0, voff = 0;
        if (MODE == MODE_GEMM) {
            voff = m * ldx * 2u + c * 16u;
            mask = m < (unsigned)a.M ? 1u : 0u;
        } else if (m < (unsigned)a.M) {
            const unsigned t = fast_div(m, a.wo_div);
            const int q = m - t * a.Wo;
            const unsigned n = fast_div(t, a.ho_div);
            const int p = t - n * a.Ho;
            const int ihc = p * a.stride, iwc = q * a.stride;
            voff = (unsigned)((n * a.H + ihc) * a.W + iwc) * ldx * 2u + c * 16u;
            // filter rows r with 0 <= ihc - pad + r < H
            const int r_lo = max(0, pad_h - ihc), r_hi = min(a.kh, a.H + pad_h - ihc);
            if (MODE == MODE_STEM) {
                mask = ((1u << r_hi) - 1u) & ~((1u << r_lo) - 1u);
                if ((unsigned)(iwc - pad_w + 2 * c) < (unsigned)a.W) mask |= 1u << 30;
                if ((unsigned)(iwc - pad_w + 2 * c + 1) < (unsigned)a.W) mask |= 1u << 31;
            } else {
                const int s_lo = max(0, pad_w - iwc), s_hi = min(a.kw, a.W + pad_w - iwc);
                const unsigned cols = ((1u << s_hi) - 1u) & ~((1u << s_lo) - 1u);
                for (int r = r_lo; r < r_hi; ++r) mask |= cols << (r * a.kw);
            }
        }
        x_voff[j] = voff;
        x_mask[j] = mask;
    }
    // Byte offset of this thread's weight chunks at slice 0, or out of bounds beyond Cout.
    unsigned w_off[W_PER];
#pragma unroll
    for (int j = 0; j < W_PER; ++j) {
        const int cid = tid + j * NT;
        const int n = n0 + cid / CPR;
        w_off[j] = n < a.Cout ? ((unsigned)n * a.K + (cid % CPR) * 8) * 2u : kOob;
    }

    // (r, s, c0) of the next K slice to load: k0 = kt*BK = (r*kwp + s)*Cin + c0.
    int fr = 0, fs = 0, fc0 = 0;
    if (MODE == MODE_STEM) {
        fr = kt0;
    } else if (MODE == MODE_GEMM) {
        fc0 = kt0 * BK;
    } else {
        const int k0 = kt0 * BK;
        const int rs = k0 / a.Cin;
        fc0 = k0 - rs * a.Cin;
        fr = rs / a.kwp;
        fs = rs - fr * a.kwp;
    }

    u32x4 rxa[PF][X_PER], rwa[PF][W_PER];

    // Issues the loads of slice kt (all zeros if kt >= kt1).  No branches; the per-load vector
    // work is one bit test and one select.  The out-of-bounds marker always travels in the
    // per-thread offset: only that operand is sure to be range-checked.
    auto load_global = [&](int kt, u32x4(&qx)[X_PER], u32x4(&qw)[W_PER]) {
        const bool live = kt < kt1;
        if (MODE == MODE_STEM) {
            // Cin == 4, kwp == 8: slice kt is filter row r = kt; chunk c holds taps 2c, 2c+1.
            const unsigned soff = (unsigned)(fr * a.W) * 8u;
            const unsigned rbit = live ? (1u << fr) : 0u;
#pragma unroll
            for (int j = 0; j < X_PER; ++j) {
                const bool row_ok = (x_mask[j] & rbit) != 0;
                const unsigned o0 = (row_ok && (x_mask[j] & (1u << 30))) ? x_voff[j] : kOob;
                const unsigned o1 = (row_ok && (x_mask[j] & (1u << 31))) ? x_voff[j] + 8u : kOob;
                const u32x2 t0 = __builtin_amdgcn_raw_buffer_load_b64(rx, o0, soff, 0);
                const u32x2 t1 = __builtin_amdgcn_raw_buffer_load_b64(rx, o1, soff, 0);
                qx[j] = u32x4{t0.x, t0.y, t1.x, t1.y};
            }
        } else {
            const unsigned soff = MODE == MODE_GEMM ? (unsigned)fc0 * 2u : ((unsigned)(fr * a.W + fs) * ldx + (unsigned)fc0) * 2u;
            const unsigned tbit = !live ? 0u : (MODE == MODE_GEMM ? 1u : (1u << (fr * a.kw + fs)));
#pragma unroll
            for (int j = 0; j < X_PER; ++j)
                qx[j] = __builtin_amdgcn_raw_buffer_load_b128(rx, (x_mask[j] & tbit) ? x_voff[j] : kOob, soff, 0);
        }
        const unsigned kb = (unsigned)kt * (BK * 2u);
#pragma unroll
        for (int j = 0; j < W_PER; ++j)
            qw[j] = __builtin_amdgcn_raw_buffer_load_b128(rw, live ? w_off[j] : kOob, kb, 0);
        if (MODE == MODE_STEM) {
            fr += 1;
        } else if (MODE == MODE_GEMM) {
            fc0 += BK;
        } else {
            fc0 += BK;
            if (fc0 == a.Cin) {
                fc0 = 0;
                if (++fs == a.kwp) { fs = 0; ++fr; }
            }
        }
    };
    auto store_lds = [&](int buf, const u32x4(&qx)[X_PER], const u32x4(&qw)[W_PER]) {
        T *sX = lds + buf * STAGE;
        T *sW = sX + BM * BK;
#pragma unroll
        for (int j = 0; j < X_PER; ++j) {
            const int cid = tid + j * NT;
            *reinterpret_cast<u32x4 *>(sX + swz<BK>(cid / CPR, cid % CPR)) = qx[j];
        }
#pragma unroll
        for (int j = 0; j < W_PER; ++j) {
            const int cid = tid + j * NT;
            *reinterpret_cast<u32x4 *>(sW + swz<BK>(cid / CPR, cid % CPR)) = qw[j];
        }
    };

    f32x16 acc[TM][TN];  // [pixel tile][channel tile]; MFMA rows = channels, columns = pixels
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // MFMAs of one K slice; operand fragments of 16-k step kk+1 are fetched from LDS while the
    // MFMAs of step kk run.
    auto compute = [&](int cur) {
        const T *sX = lds + cur * STAGE;
        const T *sW = sX + BM * BK;
        v8 fx[2][TM], fw[2][TN];
        auto fetch = [&](int kk, v8(&qx)[TM], v8(&qw)[TN]) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
                qx[i] = *reinterpret_cast<const v8 *>(sX + swz<BK>(wm0 + i * 32 + lrow, kk * 2 + lhalf));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                qw[j] = *reinterpret_cast<const v8 *>(sW + swz<BK>(wn0 + j * 32 + lrow, kk * 2 + lhalf));
        };
        fetch(0, fx[0], fw[0]);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            if (kk + 1 < BK / 16) fetch(kk + 1, fx[(kk + 1) & 1], fw[(kk + 1) & 1]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = Mfma<T>::mma(fw[kk & 1][j], fx[kk & 1][i], acc[i][j]);
        }
    };

    // Prologue: slices kt0 .. kt0+PF-1 into the register sets; the first one goes on into LDS
    // stage 0 and its set is refilled with slice kt0+PF.
#pragma unroll
    for (int u = 0; u < PF; ++u) load_global(kt0 + u, rxa[u], rwa[u]);
    store_lds(0, rxa[0], rwa[0]);
    load_global(kt0 + PF, rxa[0], rwa[0]);
    __syncthreads();

    // Steady state, PF slices per trip, no branches inside.  At the top of step kt the current
    // LDS stage holds slice kt and register set (u+1)%PF holds slice kt+1, requested PF steps
    // ago.  It is written to the other LDS stage first (every wave finished reading that stage
    // before the last barrier), the set is refilled with slice kt+1+PF, and only then do the
    // MFMAs of slice kt run, so the LDS write and the new loads sit in their shadow.
    int kt = kt0;
    int cur = 0;
    for (; kt + PF <= kt1; kt += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            store_lds(cur ^ 1, rxa[(u + 1) % PF], rwa[(u + 1) % PF]);
            load_global(kt + u + 1 + PF, rxa[(u + 1) % PF], rwa[(u + 1) % PF]);
            compute(cur);
            __syncthreads();
            cur ^= 1;
        }
    }
    // Tail: fewer than PF slices left, nothing more to load.
#pragma unroll
    for (int u = 0; u < PF - 1; ++u) {
        if (kt + u < kt1) {  // uniform across the workgroup
            if (kt + u + 1 < kt1) store_lds(cur ^ 1, rxa[(u + 1) % PF], rwa[(u + 1) % PF]);
            compute(cur);
            __syncthreads();
            cur ^= 1;
        }
    }

    const EpiPos pos{m0, n0, wm0, wn0, lrow, lhalf};
    if (SPLITK) {
        if (!splitk_exchange<TM, TN>(acc, a, pos, tile_id)) return;
    }
    // every bias and residual vector first (independent loads, one exposed latency), then the
    // arithmetic and the stores
    EpiOperands<TM, TN> eo;
    epilogue_load<TM, TN>(eo, a, pos);
    epilogue_store<T, TM, TN>(acc, eo, a, pos);
}

TileDim conv_tile_dim(ConvTile t) {
    switch (t) {
        case T128x128: return {128, 128, 256, 64, 1};
        case T128x64: return {128, 64, 256, 64, 1};
        case T64x64: return {64, 64, 256, 64, 1};
        case T64x32: return {64, 32, 128, 64, 1};
        case T32x64: return {32, 64, 128, 64, 1};
        case T128x64w2: return {128, 64, 128, 64, 1};
        case T64x128w2: return {64, 128, 128, 64, 1};
        case T256x64: return {256, 64, 256, 64, 1};
        case T128x128w8: return {128, 128, 512, 64, 1};
        case T128x64k128: return {128, 64, 256, 128, 1};
        case T64x64k128: return {64, 64, 256, 128, 1};
        case T64x32k128: return {64, 32, 128, 128, 1};
        case T32x64k128: return {32, 64, 128, 128, 1};
        case T32x32k128: return {32, 32, 64, 128, 1};
        case T128x64k128g2: return {128, 64, 512, 128, 2};
        case T64x64k128g2: return {64, 64, 512, 128, 2};
        case T64x64k128g4: return {64, 64, 1024, 128, 4};
        case T64x32k128g4: return {64, 32, 512, 128, 4};
        case T32x64k128g4: return {32, 64, 512, 128, 4};
        case T32x32k128g4: return {32, 32, 256, 128, 4};
        case T32x32k128g8: return {32, 32, 512, 128, 8};
        case T128x64g2: return {128, 64, 512, 64, 2};
        case T64x64g2: return {64, 64, 512, 64, 2};
        case T32x32g4: return {32, 32, 256, 64, 4};
        case T256x128w8: return {256, 128, 512, 64, 1};
        case T128x256w8: return {128, 256, 512, 64, 1};
        case T256x256w8: return {256, 256, 512, 64, 1};
        case T256x128: return {256, 128, 256, 64, 1};
        default: return {32, 32, 64, 64, 1};
    }
}

// The same tile with K slices of 64 (for Cin % 128 != 0), with as many wave groups as a 64-wide
// slice and the tile's thread count allow.
ConvTile conv_tile_k64(ConvTile t) {
    switch (t) {
        case T128x64k128: return T128x64;
        case T128x64k128g2: return T128x64g2;
        case T64x64k128: return T64x64;
        case T64x64k128g2: return T64x64g2;
        case T64x64k128g4: return T64x64g2;
        case T64x32k128: case T64x32k128g4: return T64x32;
        case T32x64k128: case T32x64k128g4: return T32x64;
        case T32x32k128: return T32x32;
        case T32x32k128g4: case T32x32k128g8: return T32x32g4;
        default: return t;
    }
}

// The first convolution takes the direct-to-LDS kernel's stem mode when its packed filter has 8
// rows of 8 taps x 4 channels and its stride is even (16-byte aligned 8-tap windows).
static bool stem_is_dlds(const ConvArgs &a) { return a.khp == 8 && a.kwp == 8 && a.Cin == 4 && a.stride % 2 == 0 && a.pad == 0; }

ConvTile conv_tile_staged(ConvTile t) {
    switch (t) {
        case T256x128w8: case T128x256w8: case T256x256w8: return T128x128w8;
        case T256x128: return T128x128;
        default: return conv_tile_one_group(conv_tile_k64(t));
    }
}

bool conv_uses_dlds(const ConvArgs &a, bool stem) { return stem ? stem_is_dlds(a) : a.Cin % 64 == 0; }

ConvTile conv_tile_one_group(ConvTile t) {
    switch (t) {
        case T128x64k128g2: return T128x64k128;
        case T64x64k128g2: case T64x64k128g4: return T64x64k128;
        case T64x32k128g4: return T64x32k128;
        case T32x64k128g4: return T32x64k128;
        case T32x32k128g4: case T32x32k128g8: return T32x32k128;
        case T128x64g2: return T128x64;
        case T64x64g2: return T64x64;
        case T32x32g4: return T32x32;
        default: return t;
    }
}

int conv_bk(const ConvArgs &a, bool stem, ConvTile tile) {
    if (stem) return stem_is_dlds(a) ? 64 : 32;
    if (a.Cin % 64 != 0) return 32;
    return (conv_tile_dim(tile).bk == 128 && a.Cin % 128 == 0) ? 128 : 64;
}

static bool conv_is_gemm(const ConvArgs &a, bool stem) {
    return !stem && a.kh == 1 && a.kw == 1 && a.stride == 1 && a.pad == 0 && a.Cin % 64 == 0;
}

void conv_grid(ConvTile tile, const ConvArgs &a, dim3 *grid, int *block) {
    const TileDim d = conv_tile_dim(tile);
    const unsigned tm = (a.M + d.bm - 1) / d.bm, tn = (a.Cout + d.bn - 1) / d.bn;
    *grid = dim3(tm * tn, a.split_k, a.nz > 1 ? a.nz : 1);
    *block = d.threads;
}

template <typename T, int BK, int MODE, bool SPLITK>
static hipError_t launch_conv_t(ConvTile tile, const ConvArgs &a, hipStream_t s) {
    dim3 grid;
    int block;
    tile = conv_tile_staged(tile);
    conv_grid(tile, a, &grid, &block);
    // K slices in flight in registers: 2 for the tiles with 64x64 per wave (register budget), else 3
    switch (tile) {
        case T128x128: conv_igemm_kernel<T, 128, 128, 2, 2, BK, 2, MODE, SPLITK><<<grid, block, 0, s>>>(a); break;
        case T128x64: conv_igemm_kernel<T, 128, 64, 2, 2, BK, 3, MODE, SPLITK><<<grid, block, 0, s>>>(a); break;
        case T64x64: conv_igemm_kernel<T, 64, 64, 2, 2, BK, 3, MODE, SPLITK><<<grid, block, 0, s>>>(a); break;
        case T64x32: conv_igemm_kernel<T, 64, 32, 2, 1, BK, 3, MODE, SPLITK><<<grid, block, 0, s>>>(a); break;
        case T32x64: conv_igemm_kernel<T, 32, 64, 1, 2, BK, 3, MODE, SPLITK><<<grid, block, 0, s>>>(a); break;
        case T32x32: conv_igemm_kernel<T, 32, 32, 1, 1, BK, 3, MODE, SPLITK><<<grid, block, 0, s>>>(a); break;
        case T128x64w2: conv_igemm_kernel<T, 128, 64, 2, 1, BK, 2, MODE, SPLITK><<<grid, block, 0, s>>>(a); break;
        case T64x128w2: conv_igemm_kernel<T, 64, 128, 1, 2, BK, 2, MODE, SPLITK><<<grid, block, 0, s>>>(a); break;
        case T256x64: conv_igemm_kernel<T, 256, 64, 4, 1, BK, 2, MODE, SPLITK><<<grid, block, 0, s>>>(a); break;
        case T128x128w8: conv_igemm_kernel<T, 128, 128, 2, 4, BK, 3, MODE, SPLITK><<<grid, block, 0, s>>>(a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <typename T, bool SPLITK>
static hipError_t launch_conv_dt(ConvTile tile, bool stem, const ConvArgs &a, hipStream_t s) {
    if (stem) return launch_conv_t<T, 32, MODE_STEM, SPLITK>(tile, a, s);
    return launch_conv_t<T, 32, MODE_CONV, SPLITK>(tile, a, s);
}

hipError_t launch_conv(DType dt, ConvTile tile, bool stem, const ConvArgs &a, hipStream_t s) {
    // Shapes the kernel's indexing relies on; the plan compiler guarantees them, checked again
    // here so that a bad launch is an error instead of an out-of-bounds access.
    const int bk = conv_bk(a, stem, tile);
    if (a.K % bk != 0 || a.M <= 0 || a.Cout <= 0 || a.Cout % 32 != 0 || a.split_k < 1 || a.ktiles_per_split < 1)
        return hipErrorInvalidValue;
    if (stem ? (a.Cin != 4 || a.kwp != 8 || a.khp < a.kh || a.K != a.khp * 32) : (a.Cin % 32 != 0 || a.kwp != a.kw || a.K != a.kh * a.kw * a.Cin))
        return hipErrorInvalidValue;
    if (stem ? a.kh > 30 : a.kh * a.kw > 32) return hipErrorInvalidValue;  // tap masks are 32 bits
    if ((long long)a.split_k * a.ktiles_per_split < a.K / bk) return hipErrorInvalidValue;
    if (a.split_k > 1 && (!a.partial || !a.counters)) return hipErrorInvalidValue;
    if (a.nz > 1 && (stem || !conv_is_gemm(a, stem) || a.split_k != 1 || a.bias || a.res)) return hipErrorInvalidValue;   // batched: 1x1 form only
    if (a.nz <= 1 && !a.bias) return hipErrorInvalidValue;
    if (a.split_k == 1 && a.partial) return hipErrorInvalidValue;
    // buffer descriptors address less than 2 GiB each
    if (conv_ldx(a) < a.Cin || conv_ldy(a) < a.Cout || a.Cin >= kMaxChannels || conv_ldx(a) >= kMaxChannels || conv_ldy(a) >= kMaxChannels)
        return hipErrorInvalidValue;
    if ((long long)a.B * a.H * a.W * conv_ldx(a) * 2 + (long long)(conv_pad_h(a) * a.W + conv_pad_w(a)) * conv_ldx(a) * 2 >= (1ll << 31)) return hipErrorInvalidValue;
    if ((long long)a.M * (a.partial ? a.Cout * 4ll : conv_ldy(a) * 2ll) >= (1ll << 31) || (long long)a.M * conv_ldy(a) * 2 >= (1ll << 31) || (long long)a.Cout * a.K * 2 >= (1ll << 31))
        return hipErrorInvalidValue;
    // K slices of 64 go global -> LDS directly (kernels_conv_dlds.hip); the stem and Cin % 64 != 0
    // keep the register-staged kernel of this file.
    if (stem && stem_is_dlds(a)) return launch_conv_dlds(dt, tile, bk, MODE_STEM, a, s);
    if (!stem && a.Cin % 64 == 0) return launch_conv_dlds(dt, tile, bk, conv_is_gemm(a, stem) ? MODE_GEMM : MODE_CONV, a, s);
    if (a.split_k > 1) return dt == DT_F16 ? launch_conv_dt<f16, true>(tile, stem, a, s) : launch_conv_dt<bf16, true>(tile, stem, a, s);
    return dt == DT_F16 ? launch_conv_dt<f16, false>(tile, stem, a, s) : launch_conv_dt<bf16, false>(tile, stem, a, s);
}

}  // namespace cw
