/*
 * clockwork_exec_introspect.h -- plan introspection, per-launch timing, per-layer read-back and
 * plan-compiler switches of libclockwork_exec.so.
 *
 * None of these calls is part of the paper's action model; they exist for the parity tests
 * (every kernel instantiation must be reachable and every layer comparable with the CPU
 * oracle), for the tuner that writes the plan table offline, and for the per-launch roofline
 * report.  A worker serving requests needs only clockwork_exec.h.  Same conventions as there:
 * int32_t status, [host] pointers owned by the caller, no exception crosses the boundary.
 * What they expose is the paper's "kernels per batch size" and "memory metadata" of a model
 * (section 5.1): the fixed launch list of a (model, batch) and where its tensors live.
 */
#ifndef CLOCKWORK_EXEC_INTROSPECT_H
#define CLOCKWORK_EXEC_INTROSPECT_H

#include "clockwork_exec.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Number of kernel launches in the plan of (model, batch); negative on error. */
int32_t cw_plan_num_launches(cw_ctx *ctx, int32_t model_id, int32_t batch);
typedef struct {
    int32_t op_index;      /* which op of the model this launch belongs to (fused launch: the last) */
    int32_t fused_op;      /* -1, or the op this launch computes first, fused with op_index */
    int32_t proj_op;       /* -1, or the projection-shortcut op this launch computes as well */
    int32_t pair_op;       /* -1, or a second, independent convolution over the same input computed by this launch */
    int32_t kind;          /* internal kernel family id */
    int32_t grid_x, grid_y, grid_z, block;
    int32_t tile_m, tile_n, tile_k, split_k; /* conv: pixels x channels per workgroup, K slice */
    int32_t conv_tile;     /* conv: the tile variant in cw_set_plan_override's numbering; -1 for a fused pair and for other kinds */
    int32_t wave_groups;   /* conv: groups of waves that split every K slice (1 = none) */
    int32_t next_op;       /* -1, or the 1x1 convolution over op_index's output that a fused launch computes as well (its
                              output is stored like op_index's) */
    int32_t panels;        /* conv: channel panels of the tile numbering (1 = row by row; see cw_set_panels); a pair
                              launch: of op_index's convolution in the low byte, of pair_op's in the next */
    int64_t gemm_m, gemm_n, gemm_k; /* 0 for non-GEMM launches */
    int64_t bytes;         /* algorithmic HBM bytes: inputs + weights + outputs, once each */
    int64_t flops;         /* 2 * MACs */
    char name[48];
} cw_launch_info;
int32_t cw_plan_launch_info(cw_ctx *ctx, int32_t model_id, int32_t batch, int32_t index,
                            cw_launch_info *out);
/* Runs EXEC like cw_exec but times every launch of the plan with its own pair of
 * events, issuing it `inner` (>= 1) times back to back between them (a launch is
 * idempotent); launch_us [host] receives cw_plan_num_launches() averages, each
 * including the dispatch cost of one launch.  Synchronous. */
int32_t cw_exec_timed_launches(cw_ctx *ctx, int32_t model_id, int32_t batch, int32_t slot,
                               int32_t inner, float *launch_us, void *stream);
/* Copies the output of op `op_index` from the slot's last EXEC to host_out [host]
 * as fp32 NCHW [batch][cout][h][w].  Needs the context to have been created with
 * debug retention (cw_set_debug_keep) before the plan was built; otherwise the
 * workspace region may have been reused: returns CW_ERR_UNSUPPORTED. */
int32_t cw_debug_read_op(cw_ctx *ctx, int32_t model_id, int32_t batch, int32_t op_index,
                         float *host_out, size_t capacity_floats);
/* When keep != 0, plans built afterwards give every op output its own workspace
 * region (no reuse) so cw_debug_read_op can read them.  Costs workspace only. */
int32_t cw_set_debug_keep(cw_ctx *ctx, int32_t keep);
/* EXEC normally replays, for the slot-independent middle of a plan, a HIP graph recorded at
 * LOAD (fewer, cheaper submissions; identical kernels and arguments).  on == 0 makes EXEC
 * issue every kernel as its own launch instead; on != 0 restores the default.  Takes effect
 * for the next EXEC; graphs are recorded by LOADs issued while the setting is on. */
int32_t cw_set_use_graphs(cw_ctx *ctx, int32_t on);
/* Test hook: models defined afterwards use conv tile variant `conv_tile` (0..28 =
 * 128x128, 128x64, 64x64, 64x32, 32x64, 32x32, 128x64 on 2 waves, 64x128 on 2 waves,
 * 256x64, 128x128 on 8 waves, then 128x64, 64x64, 64x32, 32x64, 32x32 with K slices of 128
 * instead of 64 (used where cin % 128 == 0, else their 64 form), then tiles whose waves come in
 * 2, 4 or 8 groups that share every K slice (128 wide: 128x64 in 2, 64x64 in 2 and 4, 64x32,
 * 32x64, 32x32 in 4, then 32x32 in 8; 64 wide: 128x64 in 2, 64x64 in 2, 32x32 in 4; the first
 * convolution takes a grouped tile's one-group form); then the tiles for large GEMMs: 256x128,
 * 128x256 and 256x256 on 8 waves, 256x128 on 4 waves (a convolution with cin % 64 != 0 takes the
 * largest basic shape below them);
 * pixels x channels per workgroup; -1 = the plan compiler's own choice)
 * and split-K factor `split_k` (0 = own choice) for every convolution, so parity
 * tests can reach every kernel instantiation.  Still fixed at plan time. */
int32_t cw_set_plan_override(cw_ctx *ctx, int32_t conv_tile, int32_t split_k);
/* A convolution with 64 or 128 output channels whose only consumer is a 1x1 stride-1
 * convolution with a residual (the last two layers of a ResNet bottleneck) is planned as ONE
 * launch when the batch gives it enough workgroups: the intermediate tensor then never leaves
 * the chip.  Where the first layer has 128 output channels (and the second a multiple of 128)
 * the launch runs two groups of four waves: they split every K slice of the first layer and
 * the channels of every chunk of the second.  on == 0 plans such pairs as two launches for models defined
 * afterwards, on == 2 as one launch of a single wave group, on == 1 restores the default;
 * other values: CW_ERR_INVALID.  Under debug retention the first layer's tensor of such a launch is
 * the one tensor that cannot be read back (it is never stored). */
int32_t cw_set_fusion(cw_ctx *ctx, int32_t on);
/* A fused launch (see above) may also compute the 1x1 stride-1 convolution that reads its output:
 * the next bottleneck's reduce, whose input then never comes back from memory.  on == 0 plans that
 * convolution as a launch of its own for models defined afterwards; on == 2 does so only where
 * the fused launch also computes a projection shortcut; on == 1 restores the default; other
 * values: CW_ERR_INVALID. */
int32_t cw_set_fusion_third(cw_ctx *ctx, int32_t on);
/* A 3x3 max pool over 64 channels whose output is the input of a 1x1 stride-1 convolution 64 -> 64
 * or 128 right behind it (ResNet-50: the first bottleneck's reduce) is planned as ONE launch with that
 * convolution when the batch gives it enough workgroups: the pooled tile goes through LDS to the
 * matrix cores and is still written for its other readers; cw_launch_info.fused_op of the max-pool
 * launch then names the convolution.  Same arithmetic, bit for bit, as the two launches.  on == 0
 * plans them as two launches for models defined afterwards (also off with cw_set_fusion(0)),
 * on != 0 restores the default. */
int32_t cw_set_fusion_pool(cw_ctx *ctx, int32_t on);
/* A depthwise 3x3 convolution without a residual whose only reader is the 1x1 stride-1 convolution right
 * behind it (a depthwise-separable block) is planned as ONE launch with that convolution for 32 or 64
 * channels into 64 or 128 when the batch gives it enough workgroups and
 * the model has no CONCAT: the depthwise result goes through LDS to the matrix cores and is never
 * stored; cw_launch_info.op_index of that launch is the 1x1, fused_op the depthwise convolution.
 * on == 0 plans them as two launches for models defined afterwards (also off with
 * cw_set_fusion(0)), on != 0 restores the default. */
int32_t cw_set_fusion_dw(cw_ctx *ctx, int32_t on);
/* Two consecutive convolutions of the plan that read the same tensor and do not depend on each
 * other (the first 1x1 of a ResNet block and the projection shortcut beside it) are planned as
 * one launch whose first workgroups compute the one and the rest the other: one dispatch and one
 * set-up latency instead of two.  Both run on one tile shape, so a member's sums may be added up
 * in another order than on its own tile (results agree to rounding).  on == 0 plans them as two launches for
 * models defined afterwards; on != 0 restores the default. */
int32_t cw_set_pair_launches(cw_ctx *ctx, int32_t on);
/* FC and SOFTMAX as one launch (up to batch 16 and 1024 classes), for models defined afterwards:
 * the FC's K is split over several workgroups per 16 outputs and the workgroup that completes the
 * last outputs computes the probabilities.  Off by default: the arrival tickets and the trips
 * through memory between the phases cost more than the second launch they save (ResNet-50 head:
 * 16.0 us against 11.8 us as two launches at batch 16, 9.8 against 9.8 at batch 1).  on == 0
 * restores the default, two launches. */
int32_t cw_set_fc_softmax(cw_ctx *ctx, int32_t on);
/* Tile numbering.  A launch's workgroups go to the chip's 8 XCDs in turn, and each XCD has an L2 of
 * its own; by default a convolution's output tiles are numbered row by row, so that an XCD
 * computes an eighth of the pixels and reads all the weights.  on != 0: for models defined
 * afterwards the plan numbers the tiles of each launch in 1, 2, 4 or 8 panels of channel tiles (an
 * XCD then reads that fraction of the weights and more of the pixels), whichever moves the fewest
 * bytes into the L2s.  Measured on ResNet-50 at batch 16: a third less traffic between the L2s and
 * the memory side over the convolution launches, and no launch faster for it (the repeats are
 * served by the last-level cache), which is why it is off by default.  Results do not depend on
 * it.  on == 0 restores the default. */
int32_t cw_set_panels(cw_ctx *ctx, int32_t on);
/* Resident launches (section 4.4: one EXEC at a time owns the whole GPU).  on != 0: plans of batch
 * sizes that are multiples of 8, compiled for models defined afterwards, run every run of plain
 * convolution layers as ONE launch of 256 workgroups that stay on their CUs: the batch is cut into
 * 8 partitions of batch/8 images, partition p is computed by the 32 workgroups on XCD p, and a
 * layer starts when the layers it reads have signalled completion through flags in the workspace
 * header, so the layers of a partition meet in one L2 and no dispatch, cache write-back or
 * invalidate separates them.  Such plans fuse and pair nothing, give every tensor its own
 * workspace region, and need the GPU to itself: every wait is bounded, and when one gives up (or a
 * workgroup finds itself on another XCD than its partition's) the EXEC still ends and
 * cw_exec_duration_ns reports CW_ERR_HIP.  CW_ERR_UNSUPPORTED on a device without 256 compute units
 * in 8 XCDs.  on == 2: only the layers of at most 4096 pixels per batch (the later stages) run that
 * way; the earlier ones keep their fused and pair launches.  on == 0 (default): one launch per
 * layer.  Other values: CW_ERR_INVALID. */
int32_t cw_set_resident(cw_ctx *ctx, int32_t on);
/* Winograd F(2x2, 3x3) (the paper's model zoo holds Winograd-compiled ResNets: Table 2).  on != 0:
 * models defined afterwards run every 3x3 stride-1 padding-1 convolution with cin % 64 == 0 as an
 * input transform, 16 GEMMs [tiles x cin] x [cin x cout] in one batched launch of the convolution
 * kernel, and an output transform with the fused epilogue: 2.25 times fewer multiply-adds, at the
 * price of two more launches, transformed tensors four times the size of the input and output, and
 * one more rounding to the storage type of the transformed input, weights and products.  LOAD
 * stores the transformed weights (16/9 of the 3x3 filter's bytes) beside the packed ones.  Such
 * convolutions are then neither fused with a following 1x1 nor paired.  on == 0 (default): the
 * direct kernel.  Applies to models defined afterwards. */
int32_t cw_set_winograd(cw_ctx *ctx, int32_t on);
/* Plan table (section 5.1: the kernels of a model are fixed per batch size ahead of time).
 * The plan compiler takes the tile variant and split-K factor of a convolution from a table
 * keyed by its GEMM shape; the library has one built in for the ResNets.  This call installs
 * `n_rows` rows that take precedence over it for models defined afterwards (n_rows == 0
 * removes them).  rows [host]: n_rows x 7 int32 = {M = batch*Ho*Wo, N = cout, K = kh*kw*cin,
 * kh, stride, conv_tile (0..28 as above), split_k >= 1}; copied.  Shapes in neither table get
 * a heuristic choice.  Plans stay a pure function of (model, batch, tables). */
int32_t cw_set_plan_table(cw_ctx *ctx, const int32_t *rows, int32_t n_rows);


#ifdef __cplusplus
}
#endif
#endif /* CLOCKWORK_EXEC_INTROSPECT_H */
