// Internal types shared by the plan compiler, the kernels and the C ABI.
// gfx950 (CDNA4) only.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace cw {

typedef _Float16 f16;
typedef __bf16 bf16;

enum DType : int32_t { DT_F16 = 0, DT_BF16 = 1 };

// Kernel families (cw_launch_info.kind).
enum Kind : int32_t {
    K_CAST_INPUT = 0,  // fp32 NCHW -> storage-type NHWC4
    K_CONV = 1,        // implicit-GEMM convolution on MFMA, fused epilogue, optional split-K
    K_MAXPOOL = 3,
    K_GAVGPOOL = 4,
    K_FC = 5,
    K_SOFTMAX = 6,
    K_DWCONV = 7,      // depthwise convolution (one filter per channel), fused epilogue
    K_COPY_CHANNELS = 8,  // a tensor into a channel range of a wider one (CONCAT sources that cannot write there themselves)
    K_WINO_INPUT = 9,   // Winograd F(2x2, 3x3): input tiles -> 16 transformed matrices
    K_WINO_OUTPUT = 10, // ... 16 product matrices -> 2x2 output tiles, fused epilogue
    K_RESIDENT = 11,    // a run of convolution layers as one launch of resident workgroups (kernels_resident.hip)
};

// Activation codes (cw_op.relu, ConvArgs.relu / relu2).
enum Act : int32_t { ACT_NONE = 0, ACT_RELU = 1, ACT_HSWISH = 2 };

// Division by a run-time constant as multiply + shifts (Granlund-Montgomery round-up method).
struct FastDiv {
    uint32_t magic, sh1, sh2;
};
inline FastDiv make_fast_div(uint32_t d) {
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;  // ceil(log2 d)
    FastDiv f;
    f.magic = (uint32_t)(((1ull << 32) * ((1ull << l) - d)) / d + 1);
    f.sh1 = l < 1 ? l : 1;
    f.sh2 = l > 0 ? l - 1 : 0;
    return f;
}

// Implicit GEMM view of a convolution (also used for the stem with Cin padded to 4 and
// the filter row padded to 8 taps): M = B*Ho*Wo output pixels, N = Cout, K = kh*kwp*Cin.
// The fields are ordered by who reads them, in runs of 64 bytes (the struct is aligned to that, and
// with it the kernel-argument segment): a workgroup's first instructions wait for every argument line
// they touch, and each further line costs a fixed fraction of a microsecond per launch.  Line 0
// is all a 1x1 stride-1 convolution without split-K reads; line 1 adds what the general
// addressing needs; split-K, the first convolution and the fused forms read on.
struct alignas(64) ConvArgs {
    // ---- line 0
    const void *x;      // NHWC [B][H][W][Cin]
    const void *w;      // packed [Cout][K], k = (r*kwp + s)*Cin + c
    const float *bias;  // [Cout]
    const void *res;    // NHWC like y, or nullptr
    void *y;            // NHWC [B][Ho][Wo][Cout]
    int32_t M, K;
    int32_t Cout, Cin;
    int32_t relu;
    int32_t nb;         // output tiles of this convolution = workgroups along x (set by the launch code)
    // ---- line 1
    int32_t B, H, W, Ho, Wo;
    int32_t kh, kw, stride;
    int32_t pad;        // padding in height | padding in width << 16 (conv_set_pad / conv_pad_h / conv_pad_w)
    FastDiv wo_div, ho_div;  // for m -> (image, row, column)
    int32_t ld;         // elements per pixel in memory: of x | of y << 16 (= Cin | Cout << 16 unless a tensor is
                        // a channel range of a wider one: CONCAT without copies); res is always dense
    // ---- line 2
    int32_t khp;        // filter rows in the packed weights (first convolution: may be padded to 8)
    int32_t split_k, ktiles_per_split;
    int32_t relu2;
    float *partial;     // split-K: [split][M][Cout] fp32, else nullptr
    int32_t *counters;  // split-K: one arrival counter per output tile, zero between launches
    // Fused second layer (launch_conv_fused only): a 1x1 stride-1 convolution over this one's
    // output, y = act2(res + bias2 + W2 * act(bias + W * x)).  `res`, `y` then belong to the second
    // layer ([M][Cout2]); the first layer's output is never stored.
    const void *w2;      // packed [Cout2][Cout]
    const float *bias2;  // [Cout2]
    int32_t Cout2;
    int32_t kwp;         // filter columns in the packed weights (first convolution: padded to 8)
    // Optional projection shortcut computed in the same launch instead of read as `res`:
    // res[m][:] = biasd + Wd * x2[m][:], x2 = [M][Cout] pixels aligned with the output (a 1x1
    // stride-1 projection of a tensor with Cout channels).  wd == nullptr: `res` is read.
    const void *x2;      // NHWC [M][Cout]
    const void *wd;      // packed [Cout2][Cout]
    const float *biasd;  // [Cout2]
    // Batched form (1x1 stride-1 addressing, no split-K): nz > 1 runs nz independent GEMMs of this
    // shape in one launch; workgroups with blockIdx.z = z take x, w and y advanced by z times these
    // byte strides (bias and res are not used then).  Read only by z > 0.
    int32_t nz;
    int32_t panel_log2;  // host side only: tile numbering of this launch (conv_pack_nb); the kernel gets it inside its tile count
    union {
        struct { long long zs_x, zs_w, zs_y; };
        // Fused form only (never batched): a third layer, the 1x1 stride-1 convolution that reads the
        // second layer's output (the next bottleneck's reduce), y3 = act3(bias3 + W3 * y), Cout3 = Cout.
        // y is still stored (it is the next block's shortcut); y3 is stored besides.  w3 == nullptr: none.
        // Together with the in-launch projection (wd) only in the one-group form.
        struct { const void *w3; const float *bias3; void *y3; };
    };
    int32_t relu3;
};
static_assert(offsetof(ConvArgs, B) == 64 && offsetof(ConvArgs, khp) == 128 && sizeof(ConvArgs) == 256, "argument lines");
// Tile numbering.  A launch's workgroups go to the 8 XCDs in turn and each XCD keeps a contiguous run
// of tile numbers, so the numbering decides what an XCD's L2 has to fetch.  Numbering 0 walks the
// tiles row by row (all channel tiles of a block of pixels, then the next pixels): every XCD reads
// an eighth of the pixels and all the weights.  Numbering p > 0 cuts the channel tiles into 2^p
// panels and walks panel after panel: an XCD reads 1/2^p of the weights and 2^p/8 of the pixels,
// which is less traffic where the weights outweigh the activations (small M, long K).  The kernel
// receives  tiles | p << 28  as its tile count (a preloaded scalar: no argument load is waited for).
constexpr int kPanelShift = 28;
__host__ __device__ inline int conv_pack_nb(int tiles, int panel_log2) { return tiles | (panel_log2 << kPanelShift); }
__host__ __device__ inline int conv_nb_tiles(int nb) { return nb & ((1 << kPanelShift) - 1); }
__host__ __device__ inline int conv_nb_panel(int nb) { return (int)((unsigned)nb >> kPanelShift); }
__host__ __device__ inline int conv_pad_h(const ConvArgs &a) { return a.pad & 0xffff; }
__host__ __device__ inline int conv_pad_w(const ConvArgs &a) { return (int)((unsigned)a.pad >> 16); }
__host__ __device__ inline int conv_ldx(const ConvArgs &a) { return a.ld & 0xffff; }
__host__ __device__ inline int conv_ldy(const ConvArgs &a) { return (int)((unsigned)a.ld >> 16); }
inline void conv_set_pad(ConvArgs &a, int pad_h, int pad_w) { a.pad = pad_h | (pad_w << 16); }
inline void conv_set_ld(ConvArgs &a, int ldx, int ldy) { a.ld = ldx | (ldy << 16); }
constexpr int kMaxChannels = 32768;  // channel counts and pitches travel in 16 bits

// Maps of at least this many pixels are averaged by the 16-wave kernel (one wave per 64 channels below).
constexpr int kGapWideFrom = 256;
// Depthwise convolution: y[m][c] = act(res[m][c] + bias[c] + sum_{r,s} x[pixel(m) + (r,s)][c] * w[r][s][c]).
struct DwArgs {
    const void *x;      // NHWC, ldx elements per pixel
    const void *w;      // packed [kh][kw][C]
    const float *bias;  // [C]
    const void *res;    // dense NHWC like y, or nullptr
    void *y;            // NHWC, ldy elements per pixel
    int32_t B, H, W, C, Ho, Wo, kh, kw, stride, pad, act, ldx, ldy;
};

// Winograd F(2x2, 3x3) for a 3x3 stride-1 pad-1 convolution.  Output pixels are cut into 2x2 tiles,
// th x tw per image (th = ceil(Ho/2), tw = ceil(Wo/2)), tiles = B*th*tw.  The input transform writes
// V[16][tiles][C]; after 16 GEMMs with the transformed weights U[16][Cout][C] (one batched launch
// of the convolution kernel), the output transform reads Mx[16][tiles][Cout] and writes y.
struct WinoArgs {
    const void *x;      // input transform: NHWC activations (ldx elements per pixel); output transform: Mx
    void *y;            // input transform: V; output transform: NHWC result (dense)
    const float *bias;  // output transform: [Cout]
    const void *res;    // output transform: dense NHWC like y, or nullptr
    int32_t B, H, W, C, th, tw, ldx, act;   // H, W: image size (= output size); C: channels of the tensor being transformed
};

// ---- resident multi-layer launch ---------------------------------------------------------------
// A run of consecutive convolution layers executed by ONE launch of 256 workgroups that stay on
// their CUs: the batch is cut into 8 partitions of B/8 images, partition p is computed by the 32
// workgroups that run on XCD p, and a layer's tiles start as soon as the tiles of the layers it reads
// (same partition, hence same XCD and same L2) have signalled completion through per-tile flags.
// Tile shapes the resident kernel holds (all on 4 waves, so that one workgroup can run any of them):
enum ResVariant : int32_t {
    RV_128x128 = 0, RV_128x64, RV_64x64, RV_128x64k128, RV_64x64k128, RV_32x32k128g4, RV_32x32g4, N_RES_VARIANTS
};
struct ResVariantDim { int bm, bn, bk; };
inline ResVariantDim res_variant_dim(int v) {
    switch (v) {
        case RV_128x128: return {128, 128, 64};
        case RV_128x64: return {128, 64, 64};
        case RV_64x64: return {64, 64, 64};
        case RV_128x64k128: return {128, 64, 128};
        case RV_64x64k128: return {64, 64, 128};
        case RV_32x32k128g4: return {32, 32, 128};
        default: return {32, 32, 64};
    }
}
// One layer of the program (device memory).  a.x, a.res and a.y hold byte offsets into the workspace
// of the tensors' first image, a.w and a.bias device addresses; partition p adds p * ps_*.
struct alignas(64) ResLayer {
    ConvArgs a;
    long long ps_x, ps_y, ps_res;
    int32_t variant;     // ResVariant; the addressing mode follows from the shape (1x1 stride 1: plain matrix)
    int32_t tiles;       // per partition
    int32_t dep[2];      // program indices of the layers that produce this layer's input and residual, or -1
    int32_t flag_base;   // this layer's first completion flag within a partition's flags
    int32_t pad_[3];
};
constexpr int kResPartitions = 8;          // = XCDs of the device
constexpr int kResGroupsPerPartition = 32; // workgroups per partition = CUs per XCD
// Workspace header behind the split-K counters: [epoch word at 0, abort word at byte 128 (holds the epoch of an
// abandoned launch), unused up to 256 B][completion flags]
constexpr size_t kResidentBytes = (size_t)1 << 20;
constexpr size_t kResidentFlagsOff = 256;
struct ResidentArgs {
    const ResLayer *layers;   // device
    int32_t n_layers;
    char *workspace;          // base the layers' activation offsets are relative to
    unsigned *flags;          // [kResPartitions][flags_per_part]
    int32_t flags_per_part;
    unsigned *epoch;          // flags equal to *epoch + 1 mean "done in this launch"
    unsigned *error;          // host-visible word: set when a wait times out or a workgroup is on the wrong XCD
    unsigned spin_limit;
};

struct CopyArgs {
    const void *src;    // [pixels][ld_src], the first C channels of every pixel are copied
    void *dst;          // [pixels][ld_dst] (already offset to the destination channel)
    int32_t pixels, C, ld_src, ld_dst;
};


struct CastArgs {
    const float *x;  // NCHW fp32 [B][C][H][W]
    void *y;         // NHWC4 [B][Hp][Wp][4]: the image inside a zero border of `pad` pixels
    int32_t B, C, H, W;
    int32_t pad, Hp, Wp;  // Hp = H + 2*pad, Wp = W + 2*pad rounded up to even
};

struct PoolArgs {
    const void *x;  // NHWC
    void *y;        // NHWC (maxpool) / fp32 [B][C] (global average)
    int32_t B, H, W, C, Ho, Wo, k, stride, pad;
};

struct FcArgs {
    const float *f;  // [B][In] fp32
    const void *w;   // [Out][In]
    const float *bias;
    float *z;        // [B][Out]
    int32_t B, In, Out;
    // FC and softmax in one launch (p != nullptr; B <= 16, Out <= 1024): K is split over split_k
    // workgroups per 16 outputs, which meet through `partial` and arrival counters like the
    // convolution's split-K; the workgroup that finishes the last 16 outputs computes p = softmax(z).
    float *p;           // [B][Out] probabilities, or nullptr: logits only (the unfused kernel)
    float *partial;     // [split_k][16][Out] fp32 (split_k > 1)
    int32_t *counters;  // ceil(Out/16) + 1 arrival counters, zero between launches
    int32_t split_k;    // 1, 2 or 4; In % (128 * split_k) == 0
};
constexpr int kFcSoftmaxMaxBatch = 16, kFcSoftmaxMaxOut = 1024;

struct SoftmaxArgs {
    const float *z;
    float *p;
    int32_t B, D;
};

// Tile shapes the conv kernel is instantiated for (fixed at plan time per layer).
// (pixels x channels per workgroup; "wN" = N waves when not 4, each wave then owning 64x64;
// "k128" = K slices of 128 instead of 64, for Cin % 128 == 0; "gN" = N groups of waves that split
// every K slice between them and add up at the end; the last four are for large GEMMs: 8 waves of
// 64x64 or 64x128 each, and 256x128 on 4 waves of 128x64)
enum ConvTile : int32_t {
    T128x128 = 0, T128x64, T64x64, T64x32, T32x64, T32x32, T128x64w2, T64x128w2, T256x64, T128x128w8,
    T128x64k128, T64x64k128, T64x32k128, T32x64k128, T32x32k128,
    T128x64k128g2, T64x64k128g2, T64x64k128g4, T64x32k128g4, T32x64k128g4, T32x32k128g4,
    T32x32k128g8, T128x64g2, T64x64g2, T32x32g4,
    T256x128w8, T128x256w8, T256x256w8, T256x128, N_CONV_TILES
};
struct TileDim {
    int bm, bn, threads, bk, kg;
};
TileDim conv_tile_dim(ConvTile t);
// The same tile with K slices of 64 (for shapes a k128 tile cannot take).
ConvTile conv_tile_k64(ConvTile t);
// The same tile with one group of waves (split-K needs that).
ConvTile conv_tile_one_group(ConvTile t);
// The largest tile of the register-staged kernel that is no larger than t (that kernel has the ten
// basic shapes only; it serves Cin % 64 != 0 and first convolutions outside the stem form).
ConvTile conv_tile_staged(ConvTile t);
// Whether a convolution runs on the direct-to-LDS kernel (else on the register-staged one).
bool conv_uses_dlds(const ConvArgs &a, bool stem);

// Launchers (kernels_*.hip).  All only enqueue; they return the launch's error state.
hipError_t launch_conv(DType dt, ConvTile tile, bool stem, const ConvArgs &a, hipStream_t s);
// The direct-to-LDS kernel for Cin % 64 == 0 and for a first convolution in its stem form
// (called by launch_conv after its checks); mode = the kernel's addressing mode.
hipError_t launch_conv_dlds(DType dt, ConvTile tile, int bk, int mode, const ConvArgs &a, hipStream_t s);
// A convolution (Cin % 64 == 0, Cout 64 or 128) and the 1x1 convolution that consumes it, in one
// launch (kernels_conv_dlds.hip).  bm = pixels per workgroup (64 or 128).
hipError_t launch_conv_fused(DType dt, int bm, int kg, const ConvArgs &a, hipStream_t s);
// Workgroups of that launch.
void conv_fused_grid(int bm, int kg, const ConvArgs &a, dim3 *grid, int *block);
bool conv_fused_ok(int bm, int kg, int cout, int cout2);   // a (pixels per workgroup, wave groups) form exists for these widths
// Two convolutions over the same input tensor in one launch (kernels_conv_dlds.hip), both on `tile`
// (one of conv_pair_tile_ok), neither split along K.
hipError_t launch_conv_pair(DType dt, ConvTile tile, const ConvArgs &a0, const ConvArgs &a1, hipStream_t s);
bool conv_pair_tile_ok(ConvTile tile);
void conv_pair_grid(ConvTile tile, const ConvArgs &a0, const ConvArgs &a1, dim3 *grid, int *block);
hipError_t launch_cast_input(DType dt, const CastArgs &a, hipStream_t s);
hipError_t launch_maxpool(DType dt, const PoolArgs &a, hipStream_t s);
hipError_t launch_gavgpool(DType dt, const PoolArgs &a, hipStream_t s);
// A 3x3 max pool over 64 channels and the 1x1 stride-1 convolution 64 -> 64 or 128 that reads it, in one launch;
// c = that convolution's arguments (its x is not read), bm = pooled pixels per workgroup (64 or 128).
hipError_t launch_maxpool_conv(DType dt, const PoolArgs &a, const ConvArgs &c, int bm, hipStream_t s);
hipError_t launch_fc(DType dt, const FcArgs &a, hipStream_t s);
hipError_t launch_softmax(const SoftmaxArgs &a, hipStream_t s);
hipError_t launch_dwconv(DType dt, const DwArgs &a, hipStream_t s);
// A depthwise 3x3 convolution over c channels (no residual) and the 1x1 stride-1 convolution c -> n that reads it, in
// one launch (channel counts of dwconv_conv_ok); cv = the 1x1's arguments (its x is not read).
hipError_t launch_dwconv_conv(DType dt, const DwArgs &a, const ConvArgs &cv, hipStream_t s);
bool dwconv_conv_ok(int c, int n);
int dwconv_conv_bm(int c, long long M);   // output pixels per workgroup of that launch
hipError_t launch_copy_channels(const CopyArgs &a, hipStream_t s);   // 2-byte elements, C % 8 == 0
hipError_t launch_resident(DType dt, const ResidentArgs &a, hipStream_t s);   // + the epoch bump behind it
// Host-side check of one program layer against what the resident kernel assumes (shapes, sizes,
// tile counts); ws_bytes = size of the workspace its offsets must stay inside.
bool resident_layer_ok(const ResLayer &l, size_t ws_bytes);
hipError_t launch_wino_input(DType dt, const WinoArgs &a, hipStream_t s);
hipError_t launch_wino_output(DType dt, const WinoArgs &a, hipStream_t s);
// LOAD-time: canonical W[cout][cin][3][3] -> U[16][cout'][cin] = G g G^T per (cout, cin), rows in the
// conv kernel's accumulator order, computed in fp32 and rounded once to the storage type
hipError_t launch_pack_winograd(DType dt, const void *src, void *dst, int cout, int cin, hipStream_t s);
// LOAD-time re-layout of depthwise weights: canonical W[C][1][kh][kw] -> [kh][kw][C]
hipError_t launch_pack_depthwise(const void *src, void *dst, int c, int kh, int kw, hipStream_t s);
// LOAD-time re-layout: canonical W[cout][cin][kh][kw] -> [cout'][khp][kwp][cinp] (zero padded);
// permute = rows in the conv kernel's MFMA accumulator order (conv weights), else plain (FC).
hipError_t launch_pack_weights(const void *src, void *dst, int cout, int cin, int kh, int kw,
                               int khp, int kwp, int cinp, bool permute, hipStream_t s);
hipError_t launch_copy_f32(const float *src, float *dst, size_t n, hipStream_t s);
// debug read-back: NHWC storage type (ld elements per pixel) -> fp32 NCHW
hipError_t launch_nhwc_to_nchw_f32(DType dt, const void *src, float *dst, int B, int C, int H,
                                   int W, int ld, hipStream_t s);
hipError_t launch_fill_zero(void *dst, size_t bytes, hipStream_t s);

// K-slice width the conv kernel uses for a shape under a tile: the tile's (128 or 64) when Cin
// is a multiple of it, else 64, else 32 (the stem and Cin % 64 != 0).
int conv_bk(const ConvArgs &a, bool stem, ConvTile tile);
// Bytes at the start of the workspace reserved for split-K arrival counters (one int per tile).
constexpr size_t kCounterBytes = 256 * 1024;
// Grid and block of a conv launch (pure function of tile and shape).
void conv_grid(ConvTile tile, const ConvArgs &a, dim3 *grid, int *block);

}  // namespace cw
