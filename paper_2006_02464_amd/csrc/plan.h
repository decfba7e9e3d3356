// Host-side model description and launch-plan compiler.
//
// A plan is the paper's "kernels per batch size" + "memory metadata" (section 5.1) for one
// (model, batch): the ordered list of kernel launches with their variant, grid, split-K factor
// and workspace offsets.  It is a pure function of (op list, input size, batch, storage type):
// nothing is measured, tuned or chosen when EXEC runs.
#pragma once
#include <string>
#include <vector>

#include "../../include/clockwork_exec_introspect.h"
#include "common.h"

namespace cw {

// Where a launch argument points; resolved to an address when EXEC is issued.
enum Space : int32_t { SP_NONE = 0, SP_WORKSPACE, SP_WEIGHTS, SP_SLOT_INPUT, SP_SLOT_LOGITS, SP_SLOT_PROBS };
struct Ref {
    Space space = SP_NONE;
    size_t offset = 0;
};

struct Launch {
    Kind kind;
    int32_t op_index;
    ConvTile tile = T64x64;
    bool stem = false;
    int32_t fused_bm = 0;  // > 0: this convolution and the 1x1 one after it in one launch (pixels per workgroup)
    int32_t fused_kg = 1;  // wave groups of that launch (1 or 2)
    // Shape fields are final; pointer fields are filled from the Refs at EXEC time.
    ConvArgs conv{};
    CastArgs cast{};
    PoolArgs pool{};
    FcArgs fc{};
    SoftmaxArgs sm{};
    DwArgs dw{};
    CopyArgs copy{};
    WinoArgs wino{};
    Ref x, w, bias, res, y, partial, counters;
    Ref probs;             // FC + softmax in one launch: the softmax's output
    Ref w2, bias2;         // second layer of a fused launch
    Ref w3, bias3, y3;     // its third layer (the next block's 1x1 reduce), when there is one
    Ref x2, wd, biasd;     // its projection shortcut, when that is computed in the launch too
    // K_MAXPOOL with pool_bm > 0: the launch also computes the 1x1 convolution info.fused_op over the pooled tensor
    // (conv = that convolution's arguments, w / bias its weights, y2 its output; pool_bm pooled pixels per workgroup)
    int32_t pool_bm = 0;
    Ref y2;
    // K_DWCONV with dw_fused: the launch computes the depthwise convolution info.fused_op (dw = its arguments, w / bias its
    // weights; its result is never stored) and the 1x1 convolution op_index over it (conv, w2 / bias2, res, y)
    bool dw_fused = false;
    // A pair launch (pair_op >= 0): a second, independent convolution over the same input tensor runs
    // in this launch's first workgroups; its arguments and tensors:
    int32_t pair_op = -1;
    ConvArgs conv0{};
    Ref w0, bias0, res0, y0;
    int64_t in_bytes = 0;  // algorithmic bytes of the input tensor (counted once in a pair)
    cw_launch_info info{};
    // K_RESIDENT: the convolution layers of the run, each with partition 0's arguments (conv), its
    // tile shape (res_variant), tiles per partition and the members it waits for; `w` of the
    // resident launch itself points at the program's place in the model's weight pages.
    std::vector<Launch> members;
    int32_t res_variant = 0, res_tiles = 0, res_dep[2] = {-1, -1}, res_flag_base = 0;
    long long res_ps_x = 0, res_ps_y = 0, res_ps_res = 0;
    int32_t res_flags_per_part = 0;
};

struct OpShape {
    int32_t c, h, w;  // output channels and spatial size
};

struct WeightSlot {        // one op that owns weights
    int32_t op_index;
    size_t blob_w_off;     // byte offset of W in the canonical blob
    size_t blob_b_off;     // byte offset of bias in the canonical blob
    size_t packed_w_off;   // byte offset of packed W inside the model's weight-pool region
    size_t packed_b_off;   // byte offset of the fp32 bias there
    size_t packed_w_bytes;
    int32_t cout, cin, kh, kw, khp, kwp, cinp;   // cin: input channels per filter (1 for a depthwise convolution)
    bool depthwise;
    size_t wino_w_off;     // Winograd-transformed weights U[16][cout][cin] (0 bytes: none)
    size_t wino_bytes;
};

struct Plan {
    int32_t batch = 0;
    std::vector<Launch> launches;
    std::vector<Ref> op_out;  // workspace (or slot) location of every op's output
    std::vector<int32_t> op_ld;  // elements from one pixel of that output to the next (> its channels where it is a
                                 // channel range of a CONCAT result)
    size_t workspace_bytes = 0;
    cw_profile profile{};
};

// Tile and split-K of one convolution GEMM shape (a row of the plan table).
struct TunedShape {
    int32_t M, N, K, kh, stride, tile, split_k;
};

struct PlanOverride {
    int32_t tile = -1;     // ConvTile or -1 = automatic
    int32_t split_k = 0;   // 0 = automatic
    bool keep_all = false; // no workspace reuse (debug read-back)
    int32_t fuse = 1;      // two-layer launches: 0 = none, 1 = yes, 2 = yes but never with two wave groups
    bool pair = true;      // two convolutions over one tensor as one launch
    bool winograd = false; // 3x3 stride-1 pad-1 convolutions through Winograd F(2x2, 3x3)
    int32_t resident = 0;  // runs of convolution layers as one launch of resident workgroups (batch % 8 == 0): 1 = every
                           // run (no fused or pair launches then), 2 = only layers of at most kResidentLateM pixels,
                           // beside the fused and pair launches of the earlier stages
    int32_t fuse_third = 1; // the next block's 1x1 reduce inside a fused 3x3 + 1x1 launch: 0 = never, 1 = yes, 2 = yes, but
                            // not in a launch that also computes a projection shortcut
    bool fc_softmax = false; // FC and softmax as one launch (batch <= 16, at most 1024 classes)
    bool fuse_pool = true;   // a 3x3 max pool over 64 channels and the 1x1 convolution 64 -> 64 or 128 that reads it as one launch
    bool fuse_dw = true;     // a depthwise 3x3 convolution and the 1x1 convolution that reads it as one launch (small channel counts)
    bool panels = false;   // tile numbering in channel panels where that moves fewer bytes into the XCDs' L2s
    std::vector<TunedShape> table;  // rows that take precedence over the built-in table
};

struct Model {
    std::vector<cw_op> ops;
    std::vector<OpShape> shapes;
    int32_t in_c = 0, in_h = 0, in_w = 0;
    DType dtype = DT_F16;
    int32_t classes = 0;
    std::vector<WeightSlot> wslots;
    std::vector<int32_t> op_wslot;  // op index -> index in wslots or -1
    size_t blob_bytes = 0;
    size_t packed_bytes = 0;   // end of the packed weights in the model's own (virtual) address range
    size_t page_bytes = 0;     // weight page size the layout was made for; no tensor straddles a multiple of it
    int32_t n_pages = 0;       // pages a LOAD takes
    std::vector<Plan> plans;
    bool keep_all = false;
    bool winograd = false;     // eligible convolutions carry transformed weights and are planned as Winograd launches
};

// Validates the op list and fills shapes, weight slots and sizes.  Returns CW_OK or an error
// with a message in *err.
int32_t model_init(Model *m, const cw_op *ops, int32_t n_ops, int32_t in_c, int32_t in_h, int32_t in_w,
                   int32_t dtype, size_t page_bytes, bool winograd, std::string *err);
// Compiles the plan of one batch size.
int32_t plan_build(const Model &m, int32_t batch, const PlanOverride &ov, Plan *out, std::string *err);
// Appends `bytes` to the model's packed layout (same page rule as the weights); returns the offset.
size_t model_reserve(Model *m, size_t bytes);
// Operator list of ResNet-18/50/152.
bool resnet_ops(int32_t depth, std::vector<cw_op> *ops);

// First-fit allocator over a fixed range (host metadata only; used for the weight pool, the
// IO cache and, at plan time, the workspace arena).
class RangeAllocator {
   public:
    explicit RangeAllocator(size_t size = 0) { reset(size); }
    void reset(size_t size);
    bool alloc(size_t bytes, size_t *offset);  // 256-byte granularity
    void free(size_t offset, size_t bytes);
    size_t free_bytes() const;
    size_t high_water() const { return high_; }

   private:
    struct Seg { size_t off, len; };
    std::vector<Seg> free_;
    size_t high_ = 0;
};

}  // namespace cw
