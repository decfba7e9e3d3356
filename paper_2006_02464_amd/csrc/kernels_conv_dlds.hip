// Per-layer launches of the direct-to-LDS implicit-GEMM convolution: kernel entry points, tile
// dispatch and the fused / pair forms.  The per-tile body is in conv_dlds_body.h.
#include "conv_dlds_body.h"

namespace cw {

template <typename T, int BM, int BN, int WARPS_M, int WARPS_N, int BK, int NS, int MODE, bool SPLITK, bool FUSED = false, int KG = 1>
__global__ __launch_bounds__(64 * WARPS_M * WARPS_N * KG) void conv_dlds_kernel(const void *x, const void *w, const void *res, void *y,
                                                                                 int M, int K, int cout_ldy, int cin_ldx, int nb, int relu,
                                                                                 const ConvArgs rest) {
    // The ten leading arguments (14 dwords, all the user SGPRs there are beside the argument
    // pointer) repeat fields of `rest`: this file is compiled with kernel-argument preloading, so
    // they are in SGPRs when a wave starts and the first address arithmetic does not wait for a
    // load of the argument block.  Everything else is read from `rest` when it is needed.
    // Cout and Cin carry the pixel pitches of y and x in their upper halves, so that the 1x1 form
    // still needs nothing beyond the preloaded scalars for its addressing.
    ConvArgs a = rest;
    a.x = x; a.w = w; a.res = res; a.y = y;
    a.M = M; a.K = K; a.Cout = cout_ldy & 0xffff; a.Cin = cin_ldx & 0xffff; a.nb = nb; a.relu = relu;
    a.ld = (int)(((unsigned)cin_ldx >> 16) | ((unsigned)cout_ldy & 0xffff0000u));
    if constexpr (MODE == MODE_GEMM && !SPLITK && !FUSED) {
        // batched form: one GEMM per blockIdx.z, operands advanced by the strides in the last argument line
        if (blockIdx.z != 0) {
            a.x = static_cast<const char *>(x) + (long long)blockIdx.z * rest.zs_x;
            a.w = static_cast<const char *>(w) + (long long)blockIdx.z * rest.zs_w;
            a.y = static_cast<char *>(y) + (long long)blockIdx.z * rest.zs_y;
        }
    }
    conv_dlds_body<T, BM, BN, WARPS_M, WARPS_N, BK, NS, MODE, SPLITK, FUSED, KG>(a, blockIdx.x, nb);
}

// Two independent convolutions that read the same tensor (the first 1x1 of a bottleneck and the
// projection shortcut beside it) in one launch: the first nb0 workgroups take the first, the rest
// the second.  Same instantiation for both (general addressing mode, no split-K); one dispatch,
// one set-up latency and one tail instead of two.
template <typename T, int BM, int BN, int WARPS_M, int WARPS_N, int BK, int NS, int KG>
__global__ __launch_bounds__(64 * WARPS_M * WARPS_N * KG) void conv_dlds_pair_kernel(const ConvArgs a0, const ConvArgs a1) {
    const int nb0 = conv_nb_tiles(a0.nb);
    if ((int)blockIdx.x < nb0)
        conv_dlds_body<T, BM, BN, WARPS_M, WARPS_N, BK, NS, MODE_CONV, false, false, KG>(a0, blockIdx.x, a0.nb);
    else
        conv_dlds_body<T, BM, BN, WARPS_M, WARPS_N, BK, NS, MODE_CONV, false, false, KG>(a1, blockIdx.x - nb0, a1.nb);
}

// A tile numbering in 2^p panels needs the channel tiles to divide evenly, and the tile count must
// leave the bits above kPanelShift free.
static bool conv_panel_ok(const ConvArgs &a, int bn, unsigned tiles) {
    if (tiles >= (1u << kPanelShift) || a.panel_log2 < 0 || a.panel_log2 > 3) return false;
    const int tiles_n = (a.Cout + bn - 1) / bn;
    return a.panel_log2 == 0 || tiles_n % (1 << a.panel_log2) == 0;
}

template <typename T, int BM, int BN, int WARPS_M, int WARPS_N, int BK, int MODE, bool SPLITK, int KG = 1>
static hipError_t launch_one(dim3 grid, int block, const ConvArgs &a_in, hipStream_t s) {
    ConvArgs a = a_in;
    if (!conv_panel_ok(a, BN, grid.x)) return hipErrorInvalidValue;
    a.nb = conv_pack_nb((int)grid.x, a.panel_log2);
    if (!SPLITK && a.ktiles_per_split != a.K / BK) return hipErrorInvalidValue;  // the kernel walks the whole K
    if (a.nz > 1 && (MODE != MODE_GEMM || SPLITK || a.bias || a.res || grid.z != (unsigned)a.nz)) return hipErrorInvalidValue;
    if (a.nz <= 1 && grid.z != 1) return hipErrorInvalidValue;
    constexpr int NS = RingDepth<BM, BN, BK>::value;
    constexpr size_t stage_bytes = (size_t)(BM + BN) * BK * 2;
    static_assert(NS * stage_bytes <= 160 * 1024, "ring does not fit the LDS");
    auto kern = conv_dlds_kernel<T, BM, BN, WARPS_M, WARPS_N, BK, NS, MODE, SPLITK, false, KG>;
    // More than 64 KiB of LDS per workgroup has to be requested once per kernel; done on first
    // use (under LOAD's graph recording or the first plain EXEC), never per launch afterwards.
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)(NS * stage_bytes));
    if (attr != hipSuccess) return attr;
    // a K walk shorter than the ring only ever touches its first stages (the wave groups' exchange
    // at the end needs its own room)
    const size_t used = std::max((size_t)std::min(NS, a.ktiles_per_split) * stage_bytes, (size_t)(KG - 1) * BM * BN * 4);
    kern<<<grid, block, used, s>>>(a.x, a.w, a.res, a.y, a.M, a.K, a.Cout | (conv_ldy(a) << 16), a.Cin | (conv_ldx(a) << 16), a.nb, a.relu, a);
    return hipGetLastError();
}

template <typename T, int MODE, bool SPLITK>
static hipError_t launch_tile(ConvTile tile, int bk, const ConvArgs &a, hipStream_t s) {
    if (MODE == MODE_STEM) tile = conv_tile_one_group(tile);
    if (bk != 128) tile = conv_tile_k64(tile);
    dim3 grid;
    int block;
    conv_grid(tile, a, &grid, &block);
    switch (tile) {
        case T128x128: return launch_one<T, 128, 128, 2, 2, 64, MODE, SPLITK>(grid, block, a, s);
        case T128x64: return launch_one<T, 128, 64, 2, 2, 64, MODE, SPLITK>(grid, block, a, s);
        case T64x64: return launch_one<T, 64, 64, 2, 2, 64, MODE, SPLITK>(grid, block, a, s);
        case T64x32: return launch_one<T, 64, 32, 2, 1, 64, MODE, SPLITK>(grid, block, a, s);
        case T32x64: return launch_one<T, 32, 64, 1, 2, 64, MODE, SPLITK>(grid, block, a, s);
        case T32x32: return launch_one<T, 32, 32, 1, 1, 64, MODE, SPLITK>(grid, block, a, s);
        case T128x64w2: return launch_one<T, 128, 64, 2, 1, 64, MODE, SPLITK>(grid, block, a, s);
        case T64x128w2: return launch_one<T, 64, 128, 1, 2, 64, MODE, SPLITK>(grid, block, a, s);
        case T256x64: return launch_one<T, 256, 64, 4, 1, 64, MODE, SPLITK>(grid, block, a, s);
        case T128x128w8: return launch_one<T, 128, 128, 2, 4, 64, MODE, SPLITK>(grid, block, a, s);
        case T128x64k128:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 128, 64, 2, 2, 128, MODE, SPLITK>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T64x64k128:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 64, 64, 2, 2, 128, MODE, SPLITK>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T64x32k128:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 64, 32, 2, 1, 128, MODE, SPLITK>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T32x64k128:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 32, 64, 1, 2, 128, MODE, SPLITK>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T32x32k128:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 32, 32, 1, 1, 128, MODE, SPLITK>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T128x64k128g2:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 128, 64, 2, 2, 128, MODE, SPLITK, 2>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T64x64k128g2:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 64, 64, 2, 2, 128, MODE, SPLITK, 2>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T64x64k128g4:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 64, 64, 2, 2, 128, MODE, SPLITK, 4>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T64x32k128g4:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 64, 32, 2, 1, 128, MODE, SPLITK, 4>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T32x64k128g4:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 32, 64, 1, 2, 128, MODE, SPLITK, 4>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T32x32k128g4:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 32, 32, 1, 1, 128, MODE, SPLITK, 4>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T32x32k128g8:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 32, 32, 1, 1, 128, MODE, SPLITK, 8>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T128x64g2:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 128, 64, 2, 2, 64, MODE, SPLITK, 2>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T64x64g2:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 64, 64, 2, 2, 64, MODE, SPLITK, 2>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T32x32g4:
            if constexpr (MODE != MODE_STEM) return launch_one<T, 32, 32, 1, 1, 64, MODE, SPLITK, 4>(grid, block, a, s);
            return hipErrorInvalidValue;
        case T256x128w8: return launch_one<T, 256, 128, 4, 2, 64, MODE, SPLITK>(grid, block, a, s);
        case T128x256w8: return launch_one<T, 128, 256, 2, 4, 64, MODE, SPLITK>(grid, block, a, s);
        case T256x256w8: return launch_one<T, 256, 256, 4, 2, 64, MODE, SPLITK>(grid, block, a, s);
        case T256x128: return launch_one<T, 256, 128, 2, 2, 64, MODE, SPLITK>(grid, block, a, s);
        default: return hipErrorInvalidValue;
    }
}

template <typename T, int BM, int BN, int MODE, int KG>
static hipError_t launch_fused_one(const ConvArgs &a_in, hipStream_t s) {
    ConvArgs a = a_in;
    a.nb = (a.M + BM - 1) / BM;
    constexpr int NS = RingDepth<BM, BN, 64>::value;
    constexpr size_t ring = (size_t)NS * (BM + BN) * 64 * 2;
    auto kern = conv_dlds_kernel<T, BM, BN, 2, 2, 64, NS, MODE, false, true, KG>;
    constexpr size_t bias_off = std::max<size_t>(ring, fused_lds_bytes(BM, BN, KG));
    static_assert(bias_off + (BN + kFusedMaxCout2 + BN) * 4 <= 160 * 1024, "fused form does not fit the LDS");
    const size_t need = bias_off + (size_t)(BN + a.Cout2 + (a.w3 ? BN : 0)) * 4;
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 (int)(bias_off + (BN + kFusedMaxCout2 + BN) * 4));
    if (attr != hipSuccess) return attr;
    if (a.Cout2 % fused_chunk(BN, KG) != 0) return hipErrorInvalidValue;
    if (a.w3 && BN / (2 * KG) < 32) return hipErrorInvalidValue;   // the third layer needs whole 32-channel tiles per wave
    kern<<<dim3((a.M + BM - 1) / BM, 1, 1), 256 * KG, need, s>>>(a.x, a.w, a.res, a.y, a.M, a.K, a.Cout | (conv_ldy(a) << 16), a.Cin | (conv_ldx(a) << 16), a.nb, a.relu, a);
    return hipGetLastError();
}

void conv_fused_grid(int bm, int kg, const ConvArgs &a, dim3 *grid, int *block) {
    *grid = dim3((a.M + bm - 1) / bm, 1, 1);
    *block = 256 * kg;
}

bool conv_fused_ok(int bm, int kg, int cout, int cout2) {
    if ((cout != 64 && cout != 128) || (bm != 64 && bm != 128) || (bm == 128 && cout == 128) || (kg != 1 && kg != 2)) return false;
    return cout2 >= cout && cout2 % fused_chunk(cout, kg) == 0 && cout2 <= kFusedMaxCout2;
}

hipError_t launch_conv_fused(DType dt, int bm, int kg, const ConvArgs &a, hipStream_t s) {
    // first layer: any convolution this kernel takes, Cout 64 or 128, whole K in one workgroup;
    // second layer: 1x1 over its output with a residual
    if (a.Cin % 64 != 0 || a.K != a.kh * a.kw * a.Cin || a.K % 64 != 0 || a.split_k != 1 || a.ktiles_per_split != a.K / 64 || a.partial)
        return hipErrorInvalidValue;
    if (!conv_fused_ok(bm, kg, a.Cout, a.Cout2)) return hipErrorInvalidValue;
    if (!a.w2 || !a.bias2) return hipErrorInvalidValue;
    if (a.wd ? (a.Cout != 64 || !a.x2 || !a.biasd) : !a.res) return hipErrorInvalidValue;
    if (!a.res && !a.wd) return hipErrorInvalidValue;
    // third layer: over the second layer's output, as many channels as the first layer has; with the projection
    // form only as one wave group (the 64-channel form is planned that way)
    if (a.w3 && ((a.wd && kg != 1) || !a.bias3 || !a.y3 || (long long)a.M * a.Cout * 2 >= (1ll << 31) || (long long)a.Cout * a.Cout2 * 2 >= (1ll << 31)))
        return hipErrorInvalidValue;
    if (a.nz > 1) return hipErrorInvalidValue;   // the batched form's strides share their place with the third layer's pointers
    if (a.kh * a.kw > 32 || (long long)a.M * a.Cout2 * 2 >= (1ll << 31) || (long long)a.Cout * a.K * 2 >= (1ll << 31)) return hipErrorInvalidValue;
    if (conv_ldx(a) != a.Cin || conv_ldy(a) != a.Cout) return hipErrorInvalidValue;   // the fused form takes dense tensors only
    if ((long long)a.B * a.H * a.W * a.Cin * 2 + (long long)(conv_pad_h(a) * a.W + conv_pad_w(a)) * a.Cin * 2 >= (1ll << 31)) return hipErrorInvalidValue;
    const bool gemm = a.kh == 1 && a.kw == 1 && a.stride == 1 && a.pad == 0;
#define CW_FUSED_T(T_, BM_, BN_, KG_) return gemm ? launch_fused_one<T_, BM_, BN_, MODE_GEMM, KG_>(a, s) : launch_fused_one<T_, BM_, BN_, MODE_CONV, KG_>(a, s)
#define CW_FUSED(BM_, BN_)                                                       \
    do {                                                                         \
        if (dt == DT_F16) {                                                      \
            if (kg == 2) { CW_FUSED_T(f16, BM_, BN_, 2); }                       \
            CW_FUSED_T(f16, BM_, BN_, 1);                                        \
        }                                                                        \
        if (kg == 2) { CW_FUSED_T(bf16, BM_, BN_, 2); }                          \
        CW_FUSED_T(bf16, BM_, BN_, 1);                                           \
    } while (0)
    if (a.Cout == 64 && bm == 128) CW_FUSED(128, 64);
    if (a.Cout == 64) CW_FUSED(64, 64);
    CW_FUSED(64, 128);
#undef CW_FUSED
#undef CW_FUSED_T
}

template <typename T, int BM, int BN, int WARPS_M, int WARPS_N, int BK, int KG>
static hipError_t launch_pair_one(const ConvArgs &a0_in, const ConvArgs &a1_in, hipStream_t s) {
    ConvArgs a0 = a0_in, a1 = a1_in;
    constexpr int NS = RingDepth<BM, BN, BK>::value;
    constexpr size_t stage_bytes = (size_t)(BM + BN) * BK * 2;
    auto kern = conv_dlds_pair_kernel<T, BM, BN, WARPS_M, WARPS_N, BK, NS, KG>;
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)(NS * stage_bytes));
    if (attr != hipSuccess) return attr;
    const size_t used = std::max((size_t)std::min(NS, std::max(a0.ktiles_per_split, a1.ktiles_per_split)) * stage_bytes, (size_t)(KG - 1) * BM * BN * 4);
    const unsigned nb0 = ((a0.M + BM - 1) / BM) * ((a0.Cout + BN - 1) / BN), nb1 = ((a1.M + BM - 1) / BM) * ((a1.Cout + BN - 1) / BN);
    if (!conv_panel_ok(a0, BN, nb0) || !conv_panel_ok(a1, BN, nb1)) return hipErrorInvalidValue;
    a0.nb = conv_pack_nb((int)nb0, a0.panel_log2);
    a1.nb = conv_pack_nb((int)nb1, a1.panel_log2);
    kern<<<dim3(nb0 + nb1, 1, 1), 64 * WARPS_M * WARPS_N * KG, used, s>>>(a0, a1);
    return hipGetLastError();
}

bool conv_pair_tile_ok(ConvTile tile) {
    switch (tile) {
        case T128x64: case T128x64k128: case T64x64: case T64x64k128: case T64x32k128: case T32x64k128: case T32x32k128:
        case T32x32k128g4: case T64x64k128g2: case T128x128: case T128x128w8: case T32x32: case T32x32g4: return true;
        default: return false;
    }
}

static bool conv_pair_member_ok(const ConvArgs &a, int bk) {
    if (a.Cin % bk != 0 || a.K != a.kh * a.kw * a.Cin || a.kwp != a.kw || a.kh * a.kw > 32 || a.split_k != 1 || a.partial) return false;
    if (a.ktiles_per_split != a.K / bk || a.M <= 0 || a.Cout % 32 != 0) return false;
    if (conv_ldx(a) < a.Cin || conv_ldy(a) < a.Cout) return false;
    if ((long long)a.B * a.H * a.W * conv_ldx(a) * 2 + (long long)(conv_pad_h(a) * a.W + conv_pad_w(a)) * conv_ldx(a) * 2 >= (1ll << 31)) return false;
    return (long long)a.M * conv_ldy(a) * 2 < (1ll << 31) && (long long)a.Cout * a.K * 2 < (1ll << 31);
}

void conv_pair_grid(ConvTile tile, const ConvArgs &a0, const ConvArgs &a1, dim3 *grid, int *block) {
    const TileDim d = conv_tile_dim(tile);
    *grid = dim3(((a0.M + d.bm - 1) / d.bm) * ((a0.Cout + d.bn - 1) / d.bn) + ((a1.M + d.bm - 1) / d.bm) * ((a1.Cout + d.bn - 1) / d.bn), 1, 1);
    *block = d.threads;
}

hipError_t launch_conv_pair(DType dt, ConvTile tile, const ConvArgs &a0, const ConvArgs &a1, hipStream_t s) {
    if (!conv_pair_tile_ok(tile)) return hipErrorInvalidValue;
    const int bk = conv_tile_dim(tile).bk;
    if (!conv_pair_member_ok(a0, bk) || !conv_pair_member_ok(a1, bk)) return hipErrorInvalidValue;
#define CW_PAIR(BM_, BN_, WM_, WN_, BK_, KG_)                                                           \
    return dt == DT_F16 ? launch_pair_one<f16, BM_, BN_, WM_, WN_, BK_, KG_>(a0, a1, s) : launch_pair_one<bf16, BM_, BN_, WM_, WN_, BK_, KG_>(a0, a1, s)
    switch (tile) {
        case T128x64: CW_PAIR(128, 64, 2, 2, 64, 1);
        case T128x64k128: CW_PAIR(128, 64, 2, 2, 128, 1);
        case T64x64: CW_PAIR(64, 64, 2, 2, 64, 1);
        case T64x64k128: CW_PAIR(64, 64, 2, 2, 128, 1);
        case T64x32k128: CW_PAIR(64, 32, 2, 1, 128, 1);
        case T32x64k128: CW_PAIR(32, 64, 1, 2, 128, 1);
        case T32x32k128: CW_PAIR(32, 32, 1, 1, 128, 1);
        case T32x32k128g4: CW_PAIR(32, 32, 1, 1, 128, 4);
        case T64x64k128g2: CW_PAIR(64, 64, 2, 2, 128, 2);
        case T128x128: CW_PAIR(128, 128, 2, 2, 64, 1);
        case T128x128w8: CW_PAIR(128, 128, 2, 4, 64, 1);
        case T32x32: CW_PAIR(32, 32, 1, 1, 64, 1);
        case T32x32g4: CW_PAIR(32, 32, 1, 1, 64, 4);
        default: return hipErrorInvalidValue;
    }
#undef CW_PAIR
}

template <typename T, bool SPLITK>
static hipError_t launch_mode(ConvTile tile, int bk, int mode, const ConvArgs &a, hipStream_t s) {
    switch (mode) {
        case MODE_GEMM: return launch_tile<T, MODE_GEMM, SPLITK>(tile, bk, a, s);
        case MODE_CONV: return launch_tile<T, MODE_CONV, SPLITK>(tile, bk, a, s);
        case MODE_STEM: return launch_tile<T, MODE_STEM, SPLITK>(tile, 64, a, s);
        default: return hipErrorInvalidValue;
    }
}

// Called by launch_conv (which has validated the shapes) for every convolution with
// Cin % 64 == 0 and for a first convolution in stem form; bk = conv_bk() of the shape under
// this tile.
hipError_t launch_conv_dlds(DType dt, ConvTile tile, int bk, int mode, const ConvArgs &a, hipStream_t s) {
    if (mode == MODE_STEM) {
        if (bk != 64 || a.Cin != 4 || a.K != 256 || a.kwp != 8 || a.khp != 8 || a.pad != 0 || a.stride % 2 != 0 || a.W % 2 != 0)
            return hipErrorInvalidValue;
        // every 8-tap window must start inside the (padded) image
        if ((a.Ho - 1) * a.stride >= a.H || (a.Wo - 1) * a.stride >= a.W) return hipErrorInvalidValue;
    } else if ((bk != 64 && bk != 128) || a.Cin % bk != 0 || a.K != a.kh * a.kw * a.Cin) {
        return hipErrorInvalidValue;
    }
    if (a.split_k > 1) return dt == DT_F16 ? launch_mode<f16, true>(tile, bk, mode, a, s) : launch_mode<bf16, true>(tile, bk, mode, a, s);
    return dt == DT_F16 ? launch_mode<f16, false>(tile, bk, mode, a, s) : launch_mode<bf16, false>(tile, bk, mode, a, s);
}

}  // namespace cw
