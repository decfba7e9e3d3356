// Model validation, weight-slot layout and the launch-plan compiler (host only).
#include "plan.h"

#include <algorithm>
#include <cstdio>
#include <cstring>

namespace cw {

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---------------------------------------------------------------- RangeAllocator
void RangeAllocator::reset(size_t size) {
    free_.clear();
    if (size) free_.push_back({0, size});
    high_ = 0;
}

bool RangeAllocator::alloc(size_t bytes, size_t *offset) {
    bytes = align_up(bytes ? bytes : 1, 256);
    for (size_t i = 0; i < free_.size(); ++i) {
        if (free_[i].len >= bytes) {
            *offset = free_[i].off;
            free_[i].off += bytes;
            free_[i].len -= bytes;
            if (free_[i].len == 0) free_.erase(free_.begin() + i);
            high_ = std::max(high_, *offset + bytes);
            return true;
        }
    }
    return false;
}

void RangeAllocator::free(size_t offset, size_t bytes) {
    bytes = align_up(bytes ? bytes : 1, 256);
    size_t i = 0;
    while (i < free_.size() && free_[i].off < offset) ++i;
    free_.insert(free_.begin() + i, {offset, bytes});
    if (i + 1 < free_.size() && free_[i].off + free_[i].len == free_[i + 1].off) {
        free_[i].len += free_[i + 1].len;
        free_.erase(free_.begin() + i + 1);
    }
    if (i > 0 && free_[i - 1].off + free_[i - 1].len == free_[i].off) {
        free_[i - 1].len += free_[i].len;
        free_.erase(free_.begin() + i);
    }
}

size_t RangeAllocator::free_bytes() const {
    size_t s = 0;
    for (const Seg &g : free_) s += g.len;
    return s;
}

// ---------------------------------------------------------------- ResNet op lists
// Post-activation ResNets with BatchNorm folded into each convolution's weights and bias; the
// stride of a down-sampling bottleneck sits on its 3x3 convolution.  A block's last conv adds
// the shortcut (the block input, or its 1x1 projection when the shape changes) before ReLU.
bool resnet_ops(int32_t depth, std::vector<cw_op> *ops) {
    int nblk[4];
    bool bottleneck;
    switch (depth) {
        case 18: nblk[0] = 2; nblk[1] = 2; nblk[2] = 2; nblk[3] = 2; bottleneck = false; break;
        case 50: nblk[0] = 3; nblk[1] = 4; nblk[2] = 6; nblk[3] = 3; bottleneck = true; break;
        case 152: nblk[0] = 3; nblk[1] = 8; nblk[2] = 36; nblk[3] = 3; bottleneck = true; break;
        default: return false;
    }
    ops->clear();
    auto add_conv = [&](int cin, int cout, int k, int stride, int pad, int relu, int src, int res) {
        cw_op o{CW_OP_CONV, cin, cout, k, k, stride, pad, relu, res, src};
        ops->push_back(o);
        return (int)ops->size() - 1;
    };
    int cur = add_conv(3, 64, 7, 2, 3, 1, -1, -1);
    ops->push_back(cw_op{CW_OP_MAXPOOL, 64, 64, 3, 3, 2, 1, 0, -1, cur});
    cur = (int)ops->size() - 1;
    int cin = 64;
    for (int stage = 0; stage < 4; ++stage) {
        const int width = 64 << stage;
        const int cout = bottleneck ? 4 * width : width;
        for (int b = 0; b < nblk[stage]; ++b) {
            const int stride = (b == 0 && stage > 0) ? 2 : 1;
            const int block_in = cur;
            int t;
            if (bottleneck) {
                t = add_conv(cin, width, 1, 1, 0, 1, block_in, -1);
                t = add_conv(width, width, 3, stride, 1, 1, t, -1);
            } else {
                t = add_conv(cin, width, 3, stride, 1, 1, block_in, -1);
            }
            int shortcut = block_in;
            if (stride != 1 || cin != cout) shortcut = add_conv(cin, cout, 1, stride, 0, 0, block_in, -1);
            cur = bottleneck ? add_conv(width, cout, 1, 1, 0, 1, t, shortcut)
                             : add_conv(width, cout, 3, 1, 1, 1, t, shortcut);
            cin = cout;
        }
    }
    ops->push_back(cw_op{CW_OP_GAVGPOOL, cin, cin, 0, 0, 1, 0, 0, -1, cur});
    ops->push_back(cw_op{CW_OP_FC, cin, 1000, 1, 1, 1, 0, 0, -1, (int)ops->size() - 1});
    ops->push_back(cw_op{CW_OP_SOFTMAX, 1000, 1000, 0, 0, 1, 0, 0, -1, (int)ops->size() - 1});
    return true;
}

// ---------------------------------------------------------------- model_init
static int32_t fail(std::string *err, int32_t code, const char *fmt, int a = 0, int b = 0) {
    char buf[256];
    snprintf(buf, sizeof buf, fmt, a, b);
    if (err) *err = buf;
    return code;
}

// A convolution the Winograd F(2x2, 3x3) path takes: 3x3, stride 1, padding 1, dense, Cin % 64 == 0.
static bool wino_eligible(const cw_op &o, int index) {
    return index > 0 && o.op == CW_OP_CONV && o.kh == 3 && o.kw == 3 && o.stride == 1 && o.pad == 1 && o.groups <= 1 && o.cin % 64 == 0 &&
           o.cout % 32 == 0;
}

int32_t model_init(Model *m, const cw_op *ops, int32_t n_ops, int32_t in_c, int32_t in_h, int32_t in_w,
                   int32_t dtype, size_t page_bytes, bool winograd, std::string *err) {
    if (!ops || n_ops < 3) return fail(err, CW_ERR_INVALID, "need at least 3 ops");
    if (dtype != CW_DTYPE_FP16 && dtype != CW_DTYPE_BF16) return fail(err, CW_ERR_INVALID, "bad dtype %d", dtype);
    if (in_c < 1 || in_h < 1 || in_w < 1) return fail(err, CW_ERR_INVALID, "bad input size");
    m->ops.assign(ops, ops + n_ops);
    m->shapes.assign(n_ops, OpShape{0, 0, 0});
    m->in_c = in_c; m->in_h = in_h; m->in_w = in_w;
    m->dtype = (DType)dtype;
    m->winograd = winograd;
    m->wslots.clear();
    m->op_wslot.assign(n_ops, -1);
    if (ops[n_ops - 2].op != CW_OP_FC || ops[n_ops - 1].op != CW_OP_SOFTMAX)
        return fail(err, CW_ERR_UNSUPPORTED, "op list must end with FC, SOFTMAX");

    size_t blob_w = 0;
    for (int i = 0; i < n_ops; ++i) {
        const cw_op &o = ops[i];
        if (o.input_from >= i || o.input_from < -1) return fail(err, CW_ERR_INVALID, "op %d: bad input_from", i);
        if ((o.input_from == -1) != (i == 0))
            return fail(err, CW_ERR_UNSUPPORTED, "op %d: only the first op may read the network input", i);
        int sc, sh, sw;
        if (o.input_from < 0) { sc = in_c; sh = in_h; sw = in_w; }
        else { sc = m->shapes[o.input_from].c; sh = m->shapes[o.input_from].h; sw = m->shapes[o.input_from].w; }
        if (o.cin != sc) return fail(err, CW_ERR_INVALID, "op %d: cin does not match its input (%d)", i, sc);
        OpShape out{o.cout, 1, 1};
        switch (o.op) {
            case CW_OP_CONV: {
                const bool dw = o.groups > 1;
                const int pad_h = o.pad, pad_w = o.kh == o.kw ? o.pad : o.pad_w;
                if (o.kh < 1 || o.kw < 1 || o.stride < 1 || pad_h < 0 || pad_w < 0 || o.relu < 0 || o.relu > 2)
                    return fail(err, CW_ERR_UNSUPPORTED, "op %d: conv needs stride >= 1, padding >= 0 and an activation code 0..2", i);
                if (dw && (o.groups != o.cin || o.cin != o.cout || o.kh != o.kw || o.cin % 8 != 0 || i == 0))
                    return fail(err, CW_ERR_UNSUPPORTED, "op %d: grouped conv must be depthwise (groups == cin == cout, %% 8, square filter)", i);
                if (sh + 2 * pad_h < o.kh || sw + 2 * pad_w < o.kw)
                    return fail(err, CW_ERR_INVALID, "op %d: filter larger than padded input", i);
                if (i == 0) {
                    if (o.cin > 4 || o.kw > 8 || o.kh != o.kw)
                        return fail(err, CW_ERR_UNSUPPORTED, "first conv needs cin<=4 and a square filter with kw<=8");
                } else if (!dw && (o.cin % 32 != 0 || o.kh * o.kw > 32)) {
                    return fail(err, CW_ERR_UNSUPPORTED, "op %d: conv needs cin %% 32 == 0 and at most 32 taps", i);
                }
                if (!dw && o.cout % 32 != 0) return fail(err, CW_ERR_UNSUPPORTED, "op %d: conv cout must be a multiple of 32", i);
                if (o.cin >= kMaxChannels || o.cout >= kMaxChannels) return fail(err, CW_ERR_UNSUPPORTED, "op %d: too many channels", i);
                out.h = (sh + 2 * pad_h - o.kh) / o.stride + 1;
                out.w = (sw + 2 * pad_w - o.kw) / o.stride + 1;
                if (o.residual_from >= 0) {
                    if (o.residual_from >= i) return fail(err, CW_ERR_INVALID, "op %d: bad residual_from", i);
                    const OpShape &r = m->shapes[o.residual_from];
                    const int rop = ops[o.residual_from].op;
                    if ((rop != CW_OP_CONV && rop != CW_OP_MAXPOOL && rop != CW_OP_CONCAT) || r.c != out.c || r.h != out.h || r.w != out.w)
                        return fail(err, CW_ERR_INVALID, "op %d: residual shape mismatch", i);
                } else if (o.residual_from != -1) {
                    return fail(err, CW_ERR_INVALID, "op %d: bad residual_from", i);
                }
                break;
            }
            case CW_OP_MAXPOOL:
                if (i == 0) return fail(err, CW_ERR_UNSUPPORTED, "first op must be a conv");
                if (o.cout != o.cin || o.cin % 8 != 0 || o.kh < 1 || o.kh != o.kw || o.stride < 1 || o.pad < 0 ||
                    o.pad >= o.kh || sh + 2 * o.pad < o.kh || sw + 2 * o.pad < o.kw)
                    return fail(err, CW_ERR_UNSUPPORTED, "op %d: unsupported max pool", i);
                out.h = (sh + 2 * o.pad - o.kh) / o.stride + 1;
                out.w = (sw + 2 * o.pad - o.kw) / o.stride + 1;
                break;
            case CW_OP_CONCAT: {
                if (i == 0 || o.residual_from < 0 || o.residual_from >= i || o.input_from < 0)
                    return fail(err, CW_ERR_INVALID, "op %d: CONCAT needs two earlier ops", i);
                const OpShape &b = m->shapes[o.residual_from];
                const int bop = ops[o.residual_from].op;
                if (bop != CW_OP_CONV && bop != CW_OP_MAXPOOL && bop != CW_OP_CONCAT)
                    return fail(err, CW_ERR_UNSUPPORTED, "op %d: CONCAT needs spatial inputs", i);
                if (b.h != sh || b.w != sw || o.cout != sc + b.c) return fail(err, CW_ERR_INVALID, "op %d: CONCAT shape mismatch", i);
                if (sc % 8 != 0 || b.c % 8 != 0 || o.cout >= kMaxChannels) return fail(err, CW_ERR_UNSUPPORTED, "op %d: CONCAT needs channel counts %% 8 == 0", i);
                out.h = sh; out.w = sw;
                break;
            }
            case CW_OP_GAVGPOOL:
                if (i == 0 || o.cout != o.cin || o.cin % 64 != 0)
                    return fail(err, CW_ERR_UNSUPPORTED, "op %d: average pool needs channels %% 64 == 0", i);
                break;
            case CW_OP_FC:
                if (i != n_ops - 2 || ops[o.input_from].op != CW_OP_GAVGPOOL || o.cin % 256 != 0 || o.cout < 1)
                    return fail(err, CW_ERR_UNSUPPORTED, "op %d: FC must follow the global average pool, cin %% 256 == 0", i);
                break;
            case CW_OP_SOFTMAX:
                if (i != n_ops - 1 || o.input_from != n_ops - 2 || o.cout != o.cin)
                    return fail(err, CW_ERR_UNSUPPORTED, "op %d: SOFTMAX must be last and read the FC", i);
                break;
            default: return fail(err, CW_ERR_INVALID, "op %d: unknown op code", i);
        }
        if (o.op != CW_OP_FC && o.op != CW_OP_SOFTMAX && o.op != CW_OP_GAVGPOOL && i > 0) {
            const int src = ops[o.input_from].op;
            if (src != CW_OP_CONV && src != CW_OP_MAXPOOL && src != CW_OP_CONCAT)
                return fail(err, CW_ERR_UNSUPPORTED, "op %d: spatial op needs a spatial input", i);
        }
        if (o.op == CW_OP_GAVGPOOL) {
            const int src = ops[o.input_from].op;
            if (src != CW_OP_CONV && src != CW_OP_MAXPOOL && src != CW_OP_CONCAT)
                return fail(err, CW_ERR_UNSUPPORTED, "op %d: average pool needs a spatial input", i);
        }
        m->shapes[i] = out;
        if (o.op == CW_OP_CONV || o.op == CW_OP_FC) {
            WeightSlot ws{};
            ws.op_index = i;
            ws.depthwise = o.op == CW_OP_CONV && o.groups > 1;
            ws.cout = o.cout; ws.cin = ws.depthwise ? 1 : o.cin;
            ws.kh = o.op == CW_OP_FC ? 1 : o.kh;
            ws.kw = o.op == CW_OP_FC ? 1 : o.kw;
            ws.kwp = (i == 0) ? 8 : ws.kw;
            ws.cinp = (i == 0) ? 4 : ws.cin;   // depthwise: [kh][kw][C], as many bytes as the canonical form
            // first convolution: with an even stride and at most 8 filter rows, the rows are padded
            // to 8 so that two of them make one K slice of 64 (see the stem mode of the conv kernel)
            ws.khp = (i == 0 && o.op == CW_OP_CONV && o.stride % 2 == 0 && ws.kh <= 8) ? 8 : ws.kh;
            ws.blob_w_off = blob_w;
            blob_w += (size_t)ws.cout * ws.cin * ws.kh * ws.kw * 2;
            m->op_wslot[i] = (int)m->wslots.size();
            m->wslots.push_back(ws);
        }
    }
    m->classes = ops[n_ops - 2].cout;
    // Packed tensors get offsets in the model's own address range, which LOAD maps page by page
    // onto whatever pages of the weight pool are free (paper section 5.1: weights live in fixed-size
    // pages): a tensor that would cross a page boundary starts on the next page instead, so every
    // tensor is contiguous in device memory wherever its page lands.  Fixed here, once, for every
    // batch size.
    if (page_bytes == 0 || page_bytes % 256 != 0) return fail(err, CW_ERR_INVALID, "weight page size must be a positive multiple of 256");
    size_t blob_b = align_up(blob_w, 4), packed = 0;
    bool too_big = false;
    auto place = [&](size_t bytes) {
        if (bytes > page_bytes) too_big = true;
        if (packed % page_bytes + bytes > page_bytes) packed = align_up(packed, page_bytes);
        const size_t at = packed;
        packed = align_up(packed + bytes, 256);
        return at;
    };
    for (WeightSlot &ws : m->wslots) {
        ws.blob_b_off = blob_b;
        blob_b += (size_t)ws.cout * 4;
        ws.packed_w_bytes = (size_t)ws.cout * ws.khp * ws.kwp * ws.cinp * 2;
        ws.packed_w_off = place(ws.packed_w_bytes);
    }
    for (WeightSlot &ws : m->wslots) ws.packed_b_off = place((size_t)ws.cout * 4);
    for (WeightSlot &ws : m->wslots) {
        ws.wino_bytes = (winograd && wino_eligible(ops[ws.op_index], ws.op_index)) ? (size_t)16 * ws.cout * ws.cin * 2 : 0;
        ws.wino_w_off = ws.wino_bytes ? place(ws.wino_bytes) : 0;
    }
    if (too_big) return fail(err, CW_ERR_UNSUPPORTED, "a weight tensor is larger than a weight page (%d bytes)", (int)page_bytes);
    m->blob_bytes = blob_b;
    m->packed_bytes = packed;
    m->page_bytes = page_bytes;
    m->n_pages = (int32_t)((packed + page_bytes - 1) / page_bytes);
    return CW_OK;
}

size_t model_reserve(Model *m, size_t bytes) {
    size_t packed = m->packed_bytes;
    if (packed % m->page_bytes + bytes > m->page_bytes) packed = align_up(packed, m->page_bytes);
    const size_t at = packed;
    m->packed_bytes = align_up(packed + bytes, 256);
    m->n_pages = (int32_t)((m->packed_bytes + m->page_bytes - 1) / m->page_bytes);
    return at;
}

// Tile shape of a layer inside a resident run: 32 workgroups share the partition's tiles in rounds,
// a tile costs about max(load-path clocks, matrix-core clocks) per K element plus a fixed part.
static int pick_res_variant(int64_t M, int64_t N, int64_t K, int32_t cin) {
    int best = RV_64x64;
    double best_cost = 1e30;
    for (int v = 0; v < N_RES_VARIANTS; ++v) {
        const ResVariantDim d = res_variant_dim(v);
        if (cin % d.bk != 0 || (d.bn > N && d.bn > 32)) continue;
        const int64_t tiles = ((M + d.bm - 1) / d.bm) * ((N + d.bn - 1) / d.bn);
        const int64_t rounds = (tiles + kResGroupsPerPartition - 1) / kResGroupsPerPartition;
        const double load_clk = (double)(d.bm + d.bn) * 2.0 / 64.0;       // bytes per K element over 64 B/clock
        const double mfma_clk = (double)d.bm * d.bn * 2.0 / 4096.0 * (d.bm <= 32 ? 2.0 : 1.0);   // small wave tiles issue at about half rate
        const double cost = (double)rounds * ((double)K * std::max(load_clk, mfma_clk) * 1.4 + 2500.0);
        if (cost < best_cost) { best_cost = cost; best = v; }
    }
    return best;
}

// ---------------------------------------------------------------- tile choice
// A measured shape takes its tile and split from the table.  Otherwise: the largest tile that
// still gives every CU at least one workgroup; below that, a 64x64 (or narrower) tile with K
// split over up to 16 workgroups.  Either way a pure function of the GEMM shape.
// Offline measurements (tune.py): the fastest tile and split-K per GEMM shape seen on an MI355X.
static const TunedShape kTuned[] = {
#include "plan_table.inc"
};

static void pick_conv_tile(int64_t M, int64_t N, int64_t K, int32_t kh, int32_t stride, int64_t ktiles,
                           const PlanOverride &ov, ConvTile *tile, int32_t *split) {
    if (ov.tile < 0 && ov.split_k <= 0) {
        auto match = [&](const TunedShape &t) {
            if (t.M != M || t.N != N || t.K != K || t.kh != kh || t.stride != stride || t.tile < 0 || t.tile >= N_CONV_TILES)
                return false;
            *tile = (ConvTile)t.tile;
            *split = (int32_t)std::max<int64_t>(1, std::min<int64_t>(t.split_k, ktiles));
            return true;
        };
        for (const TunedShape &t : ov.table)
            if (match(t)) return;
        for (const TunedShape &t : kTuned)
            if (match(t)) return;
    }
    static const ConvTile order[] = {T128x128, T128x64, T64x64, T32x64, T64x32, T32x32};
    auto blocks = [&](ConvTile t) {
        const TileDim d = conv_tile_dim(t);
        return ((M + d.bm - 1) / d.bm) * ((N + d.bn - 1) / d.bn);
    };
    const int64_t target = 256;
    ConvTile chosen = T32x32;
    bool found = false;
    for (ConvTile t : order) {
        const TileDim d = conv_tile_dim(t);
        if (d.bn > N && t != T32x32) continue;
        if (blocks(t) >= target) { chosen = t; found = true; break; }
    }
    int32_t s = 1;
    if (!found) {
        chosen = (N >= 64 && M > 32) ? T64x64 : (N >= 64 ? T32x64 : T32x32);
        const int64_t b = blocks(chosen);
        const int64_t want = (target + b - 1) / b;
        const int64_t cap = std::max<int64_t>(1, ktiles / 8);
        s = (int32_t)std::min<int64_t>(std::min(want, cap), 16);
    }
    if (ov.tile >= 0 && ov.tile < N_CONV_TILES) { chosen = (ConvTile)ov.tile; if (ov.split_k <= 0) s = 1; }
    if (ov.split_k > 0) s = (int32_t)std::min<int64_t>(ov.split_k, ktiles);
    *tile = chosen;
    *split = std::max(1, s);
}

// Tile numbering of a convolution launch (see conv_pack_nb): with 2^p channel panels each of the 8
// XCDs fetches 1/2^p of the weights and 2^p/8 of the input pixels, 8 * w_bytes / 2^p + in_bytes * 2^p
// in all; p = the count with the fewest bytes among those that divide the channel tiles evenly.
static int choose_panel(int cout, int bn, int64_t w_bytes, int64_t in_bytes) {
    const int tiles_n = (cout + bn - 1) / bn;
    int best = 0;
    int64_t best_cost = 8 * w_bytes + in_bytes;
    for (int p = 1; p <= 3 && tiles_n % (1 << p) == 0; ++p) {
        const int64_t cost = 8 * w_bytes / (1 << p) + in_bytes * (1 << p);
        if (cost < best_cost) { best_cost = cost; best = p; }
    }
    return best;
}

// ---------------------------------------------------------------- plan_build
int32_t plan_build(const Model &m, int32_t batch, const PlanOverride &ov, Plan *out, std::string *err) {
    if (batch < 1 || batch > 4096) return fail(err, CW_ERR_BAD_BATCH, "batch %d out of range", batch);
    const int n_ops = (int)m.ops.size();
    const size_t esz = 2;
    Plan p;
    p.batch = batch;
    p.op_out.assign(n_ops, Ref{});
    p.op_ld.assign(n_ops, 0);
    for (int i = 0; i < n_ops; ++i) p.op_ld[i] = m.shapes[i].c;

    // Guard the 32-bit byte offsets of the conv kernel's buffer loads (tensors stay below 2 GiB).
    {
        int64_t biggest = (int64_t)batch * m.in_h * m.in_w * 4;
        for (const OpShape &s : m.shapes) biggest = std::max<int64_t>(biggest, (int64_t)batch * s.c * s.h * s.w);
        if (biggest >= (int64_t)1 << 30) return fail(err, CW_ERR_BAD_BATCH, "batch %d: a tensor exceeds 2^30 elements", batch);
    }

    // Pairs planned as one launch: op i = a convolution with 64 or 128 output channels (Cin % 64
    // == 0, activation, no residual) whose only consumer is op j = i+1 or i+2, a 1x1 stride-1
    // convolution with a residual; enough pixels for the launch to fill the GPU.
    // Resident runs: plain convolution launches only (the layers meet in the XCD's L2 anyway), every
    // tensor in a region of its own (a tensor is written once per launch, so no cache holds an old copy).
    const int res_mode = (ov.resident && batch % kResPartitions == 0 && ov.tile < 0 && ov.split_k <= 0 && !m.winograd) ? ov.resident : 0;
    const bool resident = res_mode == 1;   // every run: plain launches only
    const bool no_reuse = ov.keep_all || res_mode != 0;
    std::vector<int> fuse_into(n_ops, -1), fused_first(n_ops, -1), fused_bm(n_ops, 0), fused_kg(n_ops, 1), proj_of(n_ops, -1);
    std::vector<int> third_of(n_ops, -1), in_third(n_ops, -1);   // fused launch of op j also computes op third_of[j]; in_third[k] = j
    if (ov.fuse && !resident && ov.tile < 0 && ov.split_k <= 0) {
        std::vector<int> uses(n_ops, 0);
        for (int i = 0; i < n_ops; ++i) {
            if (m.ops[i].input_from >= 0) ++uses[m.ops[i].input_from];
            if ((m.ops[i].op == CW_OP_CONV || m.ops[i].op == CW_OP_CONCAT) && m.ops[i].residual_from >= 0) ++uses[m.ops[i].residual_from];
        }
        for (int i = 1; i + 1 < n_ops; ++i) {
            const cw_op &o1 = m.ops[i];
            if (o1.op != CW_OP_CONV || o1.residual_from >= 0 || o1.input_from < 0 || o1.cin % 64 != 0 || uses[i] != 1) continue;
            if (o1.groups > 1 || o1.relu > 1 || m.ops[o1.input_from].op == CW_OP_CONCAT) continue;   // the fused form: dense layers, ReLU
            if (m.winograd && wino_eligible(o1, i)) continue;
            if ((o1.cout != 64 && o1.cout != 128) || o1.kh * o1.kw > 32 || o1.kh != o1.kw) continue;
            int j = -1;
            for (int t = i + 1; t <= i + 2 && t < n_ops; ++t)
                if (m.ops[t].op == CW_OP_CONV && m.ops[t].input_from == i) j = t;
            if (j < 0) continue;
            const cw_op &o2 = m.ops[j];
            if (o2.kh != 1 || o2.kw != 1 || o2.stride != 1 || o2.pad != 0 || o2.residual_from < 0 || o2.residual_from == i) continue;
            if (o2.cin != o1.cout || o2.cout % o1.cout != 0 || o2.cout > 1024 || o2.relu > 1 || o2.groups > 1) continue;
            if (m.ops[o2.residual_from].op == CW_OP_CONCAT) continue;
            const int64_t M = (int64_t)batch * m.shapes[i].h * m.shapes[i].w;
            const int bm = (o1.cout == 64 && M / 128 >= 256) ? 128 : 64;
            // measured on ResNet-50 (batch 1..16, thresholds 190, 96, 48 workgroups): 96 is as fast as 190 or 1 us
            // faster with up to 7 launches fewer; at 48 the batch-4 EXEC loses 10 us
            if ((M + bm - 1) / bm < 96) continue;
            fuse_into[i] = j; fused_first[j] = i; fused_bm[j] = bm;
            // two wave groups pay off where one workgroup per CU is all the launch has anyway (the 128-channel form)
            fused_kg[j] = (ov.fuse == 1 && o1.cout == 128 && conv_fused_ok(bm, 2, o1.cout, o2.cout)) ? 2 : 1;
            // The residual of op j may itself be a projection of a tensor as wide as op i's output
            // and aligned with it pixel for pixel (1x1, stride 1, no activation, used by nothing
            // else): then it is computed inside the launch too (64-channel form only).
            const int d = o2.residual_from;
            const cw_op &od = m.ops[d];
            if (o1.cout == 64 && od.op == CW_OP_CONV && od.kh == 1 && od.kw == 1 && od.stride == 1 && od.pad == 0 && !od.relu &&
                od.residual_from < 0 && od.input_from >= 0 && od.cin == o1.cout && od.cout == o2.cout && uses[d] == 1 && d < j &&
                fuse_into[d] < 0 && fused_first[d] < 0 && m.shapes[od.input_from].h == m.shapes[i].h &&
                m.shapes[od.input_from].w == m.shapes[i].w) {
                proj_of[j] = d;
                fuse_into[d] = j;
            }
        }
        // Third layer: the 1x1 stride-1 convolution that is the only one to read op j's output as its
        // input (the next bottleneck's reduce; the output's other reader is that block's shortcut), with
        // as many output channels as op i.
        if (ov.fuse_third) {
            std::vector<int> in_readers(n_ops, 0);
            for (int i = 0; i < n_ops; ++i)
                if (m.ops[i].op == CW_OP_CONV && m.ops[i].input_from >= 0) ++in_readers[m.ops[i].input_from];
            for (int j = 0; j + 1 < n_ops; ++j) {
                if (fused_first[j] < 0 || in_readers[j] != 1 || (proj_of[j] >= 0 && (fused_kg[j] != 1 || ov.fuse_third == 2))) continue;
                const int k = j + 1;
                const cw_op &o3 = m.ops[k];
                if (o3.op != CW_OP_CONV || o3.input_from != j || o3.kh != 1 || o3.kw != 1 || o3.stride != 1 || o3.pad != 0) continue;
                if (o3.residual_from >= 0 || o3.relu > 1 || o3.groups > 1 || o3.cin != m.ops[j].cout || o3.cout != m.ops[fused_first[j]].cout) continue;
                if (fuse_into[k] >= 0 || fused_first[k] >= 0) continue;
                bool concat_reader = false;   // its output must be a dense tensor of its own
                for (int r = k + 1; r < n_ops; ++r)
                    if (m.ops[r].op == CW_OP_CONCAT && (m.ops[r].input_from == k || m.ops[r].residual_from == k)) concat_reader = true;
                if (concat_reader) continue;
                third_of[j] = k;
                in_third[k] = j;
            }
        }
    }
    // Max pool + 1x1: a 3x3 max pool over 64 channels whose output is the input of the 1x1 stride-1
    // convolution 64 -> 64 or 128 right behind it (ResNet-50: the first bottleneck's reduce) computes that
    // convolution too, from the pooled tile in LDS, where the launch has enough workgroups; the pooled
    // tensor is still written for its other readers.
    std::vector<int> pool_conv(n_ops, -1), in_pool(n_ops, -1), pool_bm(n_ops, 0);
    if (ov.fuse && ov.fuse_pool && !resident && ov.tile < 0 && ov.split_k <= 0) {
        for (int j = 0; j + 1 < n_ops; ++j) {
            const cw_op &op = m.ops[j];
            if (op.op != CW_OP_MAXPOOL || op.kh != 3 || op.kw != 3 || m.shapes[j].c != 64) continue;
            const int k = j + 1;
            const cw_op &oc = m.ops[k];
            if (oc.op != CW_OP_CONV || oc.input_from != j || oc.kh != 1 || oc.kw != 1 || oc.stride != 1 || oc.pad != 0) continue;
            if (oc.cin != 64 || (oc.cout != 64 && oc.cout != 128) || oc.groups > 1 || oc.residual_from >= 0 || oc.relu > 1) continue;
            if (fuse_into[k] >= 0 || fused_first[k] >= 0 || in_third[k] >= 0) continue;
            bool concat_reader = false;   // its output must be a dense tensor of its own
            for (int r = k + 1; r < n_ops; ++r)
                if (m.ops[r].op == CW_OP_CONCAT && (m.ops[r].input_from == k || m.ops[r].residual_from == k)) concat_reader = true;
            if (concat_reader) continue;
            const int64_t M = (int64_t)batch * m.shapes[j].h * m.shapes[j].w;
            if (M * 8 >= ((int64_t)1 << 31) || (M + 63) / 64 < 96) continue;   // as for the fused bottleneck tails
            pool_conv[j] = k; in_pool[k] = j; pool_bm[j] = 64;
        }
    }
    // Depthwise + 1x1 (a depthwise-separable block): a depthwise 3x3 convolution without a residual whose only
    // reader is the 1x1 stride-1 convolution right behind it is computed inside that convolution's launch, from
    // LDS, for the channel counts the kernel has and where the launch has enough workgroups; models with a
    // CONCAT keep them apart (their tensors may be channel ranges of wider ones).
    std::vector<int> dw_into(n_ops, -1), dw_first(n_ops, -1);
    if (ov.fuse && ov.fuse_dw && !resident && ov.tile < 0 && ov.split_k <= 0) {
        bool has_concat = false;
        std::vector<int> uses(n_ops, 0);
        for (int i = 0; i < n_ops; ++i) {
            has_concat |= m.ops[i].op == CW_OP_CONCAT;
            if (m.ops[i].input_from >= 0) ++uses[m.ops[i].input_from];
            if ((m.ops[i].op == CW_OP_CONV || m.ops[i].op == CW_OP_CONCAT) && m.ops[i].residual_from >= 0) ++uses[m.ops[i].residual_from];
        }
        for (int i = 1; !has_concat && i + 1 < n_ops; ++i) {
            const cw_op &od = m.ops[i];
            if (od.op != CW_OP_CONV || od.groups <= 1 || od.kh != 3 || od.kw != 3 || od.residual_from >= 0 || od.input_from < 0 || uses[i] != 1) continue;
            const int k = i + 1;
            const cw_op &oc = m.ops[k];
            if (oc.op != CW_OP_CONV || oc.groups > 1 || oc.input_from != i || oc.residual_from == i) continue;
            if (oc.kh != 1 || oc.kw != 1 || oc.stride != 1 || oc.pad != 0 || oc.cin != od.cout || !dwconv_conv_ok(od.cout, oc.cout)) continue;
            if (fuse_into[k] >= 0 || fused_first[k] >= 0 || in_third[k] >= 0 || in_pool[k] >= 0) continue;
            const int64_t M = (int64_t)batch * m.shapes[i].h * m.shapes[i].w;
            if (M * 16 >= ((int64_t)1 << 31) || (M + 63) / 64 < 96) continue;
            dw_into[i] = k; dw_first[k] = i;
        }
    }
    // Order in which the ops are planned and launched: op order, except that a convolution j which
    // reads the same tensor as an earlier convolution i and depends on nothing after i (a ResNet
    // block's projection shortcut, i = the block's first 1x1) moves to right behind i, where the two
    // become one launch (below).
    std::vector<int> order;
    {
        std::vector<char> moved(n_ops, 0);
        std::vector<int> partner(n_ops, -1);
        if (ov.pair && !resident && ov.tile < 0 && ov.split_k <= 0) {
            for (int i = 1; i < n_ops; ++i) {
                const cw_op &a = m.ops[i];
                if (a.op != CW_OP_CONV || a.groups > 1 || a.input_from < 0 || a.cin % 64 != 0 || fuse_into[i] >= 0 || fused_first[i] >= 0 || moved[i]) continue;
                if (in_third[i] >= 0 || in_pool[i] >= 0 || dw_first[i] >= 0) continue;
                if (m.winograd && wino_eligible(a, i)) continue;
                for (int j = i + 1; j < n_ops && j <= i + 3; ++j) {
                    const cw_op &b = m.ops[j];
                    if (b.op != CW_OP_CONV || b.groups > 1 || b.input_from != a.input_from || fuse_into[j] >= 0 || fused_first[j] >= 0 || moved[j] || in_third[j] >= 0 || in_pool[j] >= 0 || dw_first[j] >= 0) continue;
                    if (b.residual_from >= i || (m.winograd && wino_eligible(b, j))) continue;
                    partner[i] = j; moved[j] = 1;
                    break;
                }
            }
        }
        for (int i = 0; i < n_ops; ++i) {
            if (moved[i]) continue;
            order.push_back(i);
            if (partner[i] >= 0) order.push_back(partner[i]);
        }
    }
    std::vector<int> pos(n_ops);
    for (int t = 0; t < n_ops; ++t) pos[order[t]] = t;
    // Time (position in `order`) of the last read of every op's output.  An op computed inside a
    // fused launch reads its inputs when that launch runs.
    std::vector<int> last_use(n_ops, -1);
    for (int i = 0; i < n_ops; ++i) {
        const int at = pos[fuse_into[i] >= 0 ? fuse_into[i] : (in_third[i] >= 0 ? in_third[i] : (in_pool[i] >= 0 ? in_pool[i] : (dw_into[i] >= 0 ? dw_into[i] : i)))];
        if (m.ops[i].input_from >= 0) last_use[m.ops[i].input_from] = std::max(last_use[m.ops[i].input_from], at);
        if ((m.ops[i].op == CW_OP_CONV || m.ops[i].op == CW_OP_CONCAT) && m.ops[i].residual_from >= 0)
            last_use[m.ops[i].residual_from] = std::max(last_use[m.ops[i].residual_from], at);
    }
    // CONCAT without copies: a source that is a convolution (or another CONCAT) whose every other
    // reader can follow a pixel pitch (a convolution reading it as its input) gets its place inside
    // the CONCAT's tensor and writes there itself: host[s] = the CONCAT, choff[s] = its first
    // channel there.  Chains (a CONCAT that is the first source of the next, as in a dense block)
    // resolve to the last CONCAT's tensor; every member is then a channel range of it with that
    // tensor's pitch.  Sources that do not qualify are copied in by a launch of their own.
    std::vector<int> host(n_ops, -1), choff(n_ops, 0);
    {
        std::vector<std::vector<int>> readers(n_ops);
        for (int i = 0; i < n_ops; ++i) {
            if (m.ops[i].input_from >= 0) readers[m.ops[i].input_from].push_back(i);
            if ((m.ops[i].op == CW_OP_CONV || m.ops[i].op == CW_OP_CONCAT) && m.ops[i].residual_from >= 0) readers[m.ops[i].residual_from].push_back(i);
        }
        for (int c = 1; c < n_ops; ++c) {
            if (m.ops[c].op != CW_OP_CONCAT) continue;
            const int src[2] = {m.ops[c].input_from, m.ops[c].residual_from};
            const int at[2] = {0, m.shapes[src[0]].c};
            for (int k = 0; k < 2; ++k) {
                const int sidx = src[k];
                if (k == 1 && sidx == src[0]) continue;
                const cw_op &so = m.ops[sidx];
                if ((so.op != CW_OP_CONV && so.op != CW_OP_CONCAT) || host[sidx] >= 0 || fuse_into[sidx] >= 0 || fused_first[sidx] >= 0) continue;
                if (m.winograd && wino_eligible(so, sidx)) continue;   // its output transform writes dense tensors only
                bool ok = true;
                for (int u : readers[sidx]) {
                    if (u == c) continue;
                    const cw_op &uo = m.ops[u];
                    if (uo.op == CW_OP_CONCAT) continue;   // that one copies (this source has its host already)
                    if (uo.op == CW_OP_CONV && uo.input_from == sidx && uo.residual_from != sidx && fuse_into[u] < 0 && fused_first[u] < 0) continue;
                    ok = false;
                }
                if (ok) { host[sidx] = c; choff[sidx] = at[k]; }
            }
        }
    }
    auto root_of = [&](int i) { while (host[i] >= 0) i = host[i]; return i; };
    auto offset_in_root = [&](int i) { int o = 0; while (host[i] >= 0) { o += choff[i]; i = host[i]; } return o; };
    for (int i = 0; i < n_ops; ++i) {   // a hosting tensor lives as long as anything inside it is read
        const int r = root_of(i);
        if (r != i) last_use[r] = std::max(last_use[r], std::max(last_use[i], pos[r]));
    }
    std::vector<long long> root_off(n_ops, -1);
    std::vector<size_t> out_bytes(n_ops, 0);
    RangeAllocator arena((size_t)1 << 46);
    auto ws_alloc = [&](size_t bytes) {
        size_t off = 0;
        arena.alloc(bytes, &off);
        return off;
    };

    // Where op i's output goes: a region of its own, or its channel range of the CONCAT tensor
    // that hosts it (allocated when its first member is planned).
    auto place_output = [&](int i, size_t dense_bytes) {
        const int r = root_of(i);
        if (r == i && root_off[i] < 0) {
            out_bytes[i] = dense_bytes;
            p.op_out[i] = Ref{SP_WORKSPACE, ws_alloc(dense_bytes)};
            return;
        }
        const OpShape &rs = m.shapes[r];
        const size_t root_bytes = (size_t)batch * rs.h * rs.w * rs.c * esz;
        if (root_off[r] < 0) root_off[r] = (long long)ws_alloc(root_bytes);
        p.op_out[i] = Ref{SP_WORKSPACE, (size_t)root_off[r] + (size_t)offset_in_root(i) * esz};
        p.op_ld[i] = rs.c;
        out_bytes[i] = r == i ? root_bytes : 0;   // members are never freed on their own
    };

    // the split-K arrival counters live at the very start of the workspace, never reused; behind
    // them the epoch word and completion flags of resident launches
    (void)ws_alloc(kCounterBytes);
    (void)ws_alloc(kResidentBytes);

    // input cast: fp32 NCHW in the IO slot -> NHWC4 in the workspace, inside a zero border as wide
    // as the first convolution's padding (that convolution then runs unpadded over the larger image)
    const int in_pad = m.ops[0].op == CW_OP_CONV ? m.ops[0].pad : 0;
    const int in_hp = m.in_h + 2 * in_pad, in_wp = (m.in_w + 2 * in_pad + 1) / 2 * 2;
    const size_t cast_bytes = (size_t)batch * in_hp * in_wp * 4 * esz;
    const size_t cast_off = ws_alloc(cast_bytes);
    {
        Launch l{};
        l.kind = K_CAST_INPUT;
        l.op_index = 0;
        l.cast.B = batch; l.cast.C = m.in_c; l.cast.H = m.in_h; l.cast.W = m.in_w;
        l.cast.pad = in_pad; l.cast.Hp = in_hp; l.cast.Wp = in_wp;
        l.x = Ref{SP_SLOT_INPUT, 0};
        l.y = Ref{SP_WORKSPACE, cast_off};
        l.info.bytes = (int64_t)batch * m.in_c * m.in_h * m.in_w * 4 + (int64_t)cast_bytes;
        snprintf(l.info.name, sizeof l.info.name, "cast_input");
        p.launches.push_back(l);
    }

    for (int t = 0; t < n_ops; ++t) {
        const int i = order[t];
        const cw_op &o = m.ops[i];
        const OpShape &os = m.shapes[i];
        int sc, sh, sw;
        Ref src;
        if (o.input_from < 0) { sc = 4; sh = m.in_h; sw = m.in_w; src = Ref{SP_WORKSPACE, cast_off}; }  // logical size; see below
        else { sc = m.shapes[o.input_from].c; sh = m.shapes[o.input_from].h; sw = m.shapes[o.input_from].w; src = p.op_out[o.input_from]; }
        size_t partial_off = 0, partial_bytes = 0;
        size_t tmp_off[2] = {0, 0}, tmp_bytes[2] = {0, 0};   // Winograd: transformed input and products

        switch (o.op) {
            case CW_OP_CONV: {
                const WeightSlot &ws = m.wslots[m.op_wslot[i]];
                if (fuse_into[i] >= 0) break;  // computed inside the launch of op fuse_into[i]; its output is never stored
                if (in_third[i] >= 0) break;   // computed, and its output placed, by the fused launch of op in_third[i]
                if (in_pool[i] >= 0) break;    // likewise by the max-pool launch of op in_pool[i]
                if (dw_into[i] >= 0) break;    // a depthwise convolution computed inside the launch of the 1x1 behind it; never stored
                if (fused_first[i] >= 0) {
                    const int f = fused_first[i];
                    const cw_op &o1 = m.ops[f];
                    const OpShape &s1 = m.shapes[f];
                    const OpShape &sin = m.shapes[o1.input_from];
                    const WeightSlot &ws1 = m.wslots[m.op_wslot[f]];
                    out_bytes[i] = (size_t)batch * os.h * os.w * os.c * esz;
                    p.op_out[i] = Ref{SP_WORKSPACE, ws_alloc(out_bytes[i])};
                    Launch l{};
                    l.kind = K_CONV;
                    l.op_index = i;
                    l.fused_bm = fused_bm[i];
                    l.fused_kg = fused_kg[i];
                    ConvArgs &a = l.conv;
                    a.B = batch; a.H = sin.h; a.W = sin.w; a.Cin = o1.cin; a.Ho = s1.h; a.Wo = s1.w; a.Cout = o1.cout;
                    a.kh = o1.kh; a.kw = o1.kw; a.kwp = o1.kw; a.khp = o1.kh; a.stride = o1.stride;
                    conv_set_pad(a, o1.pad, o1.kh == o1.kw ? o1.pad : o1.pad_w);
                    conv_set_ld(a, o1.cin, o1.cout);
                    a.M = batch * s1.h * s1.w;
                    a.K = o1.kh * o1.kw * o1.cin;
                    a.relu = o1.relu;
                    a.split_k = 1; a.ktiles_per_split = a.K / 64;
                    a.wo_div = make_fast_div((uint32_t)s1.w);
                    a.ho_div = make_fast_div((uint32_t)s1.h);
                    a.Cout2 = o.cout; a.relu2 = o.relu;
                    l.x = p.op_out[o1.input_from];
                    l.w = Ref{SP_WEIGHTS, ws1.packed_w_off};
                    l.bias = Ref{SP_WEIGHTS, ws1.packed_b_off};
                    l.w2 = Ref{SP_WEIGHTS, ws.packed_w_off};
                    l.bias2 = Ref{SP_WEIGHTS, ws.packed_b_off};
                    l.y = p.op_out[i];
                    const int64_t in_pixels = (o1.kh == 1 && o1.stride > 1) ? (int64_t)a.M : (int64_t)batch * sin.h * sin.w;
                    l.info.fused_op = f;
                    l.info.proj_op = proj_of[i];
                    l.info.gemm_m = a.M; l.info.gemm_n = a.Cout; l.info.gemm_k = a.K;
                    l.info.flops = 2 * (int64_t)a.M * a.Cout * a.K + 2 * (int64_t)a.M * o.cout * o.cin;
                    l.info.bytes = in_pixels * o1.cin * esz + ((int64_t)o1.cout * a.K + (int64_t)o.cout * o.cin) * esz + (o1.cout + o.cout) * 4 +
                                   (int64_t)out_bytes[i];
                    if (proj_of[i] >= 0) {
                        const int d = proj_of[i];
                        const WeightSlot &wsd = m.wslots[m.op_wslot[d]];
                        l.x2 = p.op_out[m.ops[d].input_from];
                        l.wd = Ref{SP_WEIGHTS, wsd.packed_w_off};
                        l.biasd = Ref{SP_WEIGHTS, wsd.packed_b_off};
                        l.info.flops += 2 * (int64_t)a.M * m.ops[d].cout * m.ops[d].cin;
                        l.info.bytes += (int64_t)a.M * m.ops[d].cin * esz + (int64_t)m.ops[d].cout * m.ops[d].cin * esz + m.ops[d].cout * 4;
                        snprintf(l.info.name, sizeof l.info.name, "conv%dx%d_s%d+1x1+proj", o1.kh, o1.kw, o1.stride);
                    } else {
                        l.res = p.op_out[o.residual_from];
                        l.info.bytes += (int64_t)out_bytes[i];   // the residual tensor
                        snprintf(l.info.name, sizeof l.info.name, "conv%dx%d_s%d+1x1", o1.kh, o1.kw, o1.stride);
                    }
                    l.info.next_op = -1;
                    if (third_of[i] >= 0) {
                        const int k = third_of[i];
                        const cw_op &o3 = m.ops[k];
                        const WeightSlot &ws3 = m.wslots[m.op_wslot[k]];
                        out_bytes[k] = (size_t)batch * os.h * os.w * o3.cout * esz;
                        p.op_out[k] = Ref{SP_WORKSPACE, ws_alloc(out_bytes[k])};
                        p.op_ld[k] = o3.cout;
                        a.relu3 = o3.relu;
                        l.w3 = Ref{SP_WEIGHTS, ws3.packed_w_off};
                        l.bias3 = Ref{SP_WEIGHTS, ws3.packed_b_off};
                        l.y3 = p.op_out[k];
                        l.info.next_op = k;
                        l.info.flops += 2 * (int64_t)a.M * o3.cout * o3.cin;
                        l.info.bytes += (int64_t)o3.cout * o3.cin * esz + o3.cout * 4 + (int64_t)out_bytes[k];   // its input never leaves the chip
                        const size_t len = strlen(l.info.name);
                        snprintf(l.info.name + len, sizeof l.info.name - len, "+1x1");
                    }
                    l.info.tile_m = l.fused_bm; l.info.tile_n = a.Cout; l.info.tile_k = 64; l.info.split_k = 1;
                    l.info.conv_tile = -1; l.info.wave_groups = l.fused_kg;
                    p.launches.push_back(l);
                    break;
                }
                place_output(i, (size_t)batch * os.h * os.w * os.c * esz);
                if (dw_first[i] >= 0) {   // the depthwise convolution in front of this 1x1, and the 1x1, as one launch
                    const int f = dw_first[i];
                    const cw_op &od = m.ops[f];
                    const OpShape &sd = m.shapes[f];
                    const OpShape &sin = m.shapes[od.input_from];
                    const WeightSlot &wsd = m.wslots[m.op_wslot[f]];
                    Launch l{};
                    l.kind = K_DWCONV;
                    l.op_index = i;
                    l.dw_fused = true;
                    l.dw = DwArgs{nullptr, nullptr, nullptr, nullptr, nullptr, batch, sin.h, sin.w, od.cin, sd.h, sd.w, od.kh, od.kw, od.stride, od.pad,
                                  od.relu, p.op_ld[od.input_from], od.cout};
                    ConvArgs &a = l.conv;
                    a.B = batch; a.H = sd.h; a.W = sd.w; a.Cin = o.cin; a.Ho = os.h; a.Wo = os.w; a.Cout = o.cout;
                    a.kh = 1; a.kw = 1; a.kwp = 1; a.khp = 1; a.stride = 1;
                    conv_set_pad(a, 0, 0);
                    conv_set_ld(a, o.cin, p.op_ld[i]);
                    a.M = batch * os.h * os.w;
                    a.K = o.cin;
                    a.relu = o.relu;
                    a.split_k = 1; a.ktiles_per_split = 1;
                    l.x = p.op_out[od.input_from];
                    l.w = Ref{SP_WEIGHTS, wsd.packed_w_off};
                    l.bias = Ref{SP_WEIGHTS, wsd.packed_b_off};
                    l.w2 = Ref{SP_WEIGHTS, ws.packed_w_off};
                    l.bias2 = Ref{SP_WEIGHTS, ws.packed_b_off};
                    l.y = p.op_out[i];
                    if (o.residual_from >= 0) l.res = p.op_out[o.residual_from];
                    const int64_t out_b = (int64_t)batch * os.h * os.w * os.c * esz;
                    l.info.fused_op = f;
                    l.info.gemm_m = a.M; l.info.gemm_n = a.Cout; l.info.gemm_k = a.K;
                    l.info.flops = 2 * (int64_t)a.M * od.cout * od.kh * od.kw + 2 * (int64_t)a.M * a.Cout * a.K;
                    l.info.bytes = (int64_t)batch * sin.h * sin.w * sin.c * esz + (int64_t)od.cout * od.kh * od.kw * esz + od.cout * 4 +
                                   (int64_t)o.cout * o.cin * esz + o.cout * 4 + out_b + (o.residual_from >= 0 ? out_b : 0);
                    snprintf(l.info.name, sizeof l.info.name, "dwconv%dx%d_s%d+1x1", od.kh, od.kw, od.stride);
                    p.launches.push_back(l);
                    break;
                }
                if (o.groups > 1) {   // depthwise: its own kernel
                    Launch l{};
                    l.kind = K_DWCONV;
                    l.op_index = i;
                    l.dw = DwArgs{nullptr, nullptr, nullptr, nullptr, nullptr, batch, sh, sw, o.cin, os.h, os.w, o.kh, o.kw, o.stride, o.pad,
                                  o.relu, p.op_ld[o.input_from], p.op_ld[i]};
                    l.x = src;
                    l.w = Ref{SP_WEIGHTS, ws.packed_w_off};
                    l.bias = Ref{SP_WEIGHTS, ws.packed_b_off};
                    l.y = p.op_out[i];
                    if (o.residual_from >= 0) l.res = p.op_out[o.residual_from];
                    const int64_t out_b = (int64_t)batch * os.h * os.w * os.c * esz;
                    l.info.flops = 2 * (int64_t)batch * os.h * os.w * os.c * o.kh * o.kw;
                    l.info.bytes = (int64_t)batch * sh * sw * sc * esz + (int64_t)o.cout * o.kh * o.kw * esz + o.cout * 4 + out_b + (o.residual_from >= 0 ? out_b : 0);
                    snprintf(l.info.name, sizeof l.info.name, "dwconv%dx%d_s%d", o.kh, o.kw, o.stride);
                    p.launches.push_back(l);
                    break;
                }
                if (m.winograd && ws.wino_bytes && ov.tile < 0 && ov.split_k <= 0) {
                    // Winograd F(2x2, 3x3): input transform, 16 GEMMs [tiles x Cin] x [Cin x Cout] as one
                    // batched launch of the convolution kernel, output transform with the fused epilogue.
                    const int th = (os.h + 1) / 2, tw = (os.w + 1) / 2;
                    const int64_t tiles = (int64_t)batch * th * tw;
                    tmp_bytes[0] = (size_t)16 * tiles * o.cin * esz;
                    tmp_bytes[1] = (size_t)16 * tiles * o.cout * esz;
                    tmp_off[0] = ws_alloc(tmp_bytes[0]);
                    tmp_off[1] = ws_alloc(tmp_bytes[1]);
                    Launch li{};
                    li.kind = K_WINO_INPUT;
                    li.op_index = i;
                    li.wino = WinoArgs{nullptr, nullptr, nullptr, nullptr, batch, sh, sw, o.cin, th, tw, p.op_ld[o.input_from], 0};
                    li.x = src;
                    li.y = Ref{SP_WORKSPACE, tmp_off[0]};
                    li.info.bytes = (int64_t)batch * sh * sw * o.cin * esz + (int64_t)tmp_bytes[0];
                    snprintf(li.info.name, sizeof li.info.name, "winograd_input");
                    p.launches.push_back(li);
                    Launch lg{};
                    lg.kind = K_CONV;
                    lg.op_index = i;
                    ConvArgs &g = lg.conv;
                    g.B = 1; g.H = 1; g.W = (int32_t)tiles; g.Ho = 1; g.Wo = (int32_t)tiles; g.Cin = o.cin; g.Cout = o.cout;
                    g.kh = 1; g.kw = 1; g.kwp = 1; g.khp = 1; g.stride = 1; g.pad = 0;
                    conv_set_ld(g, o.cin, o.cout);
                    g.M = (int32_t)tiles; g.K = o.cin; g.relu = 0;
                    g.wo_div = make_fast_div((uint32_t)tiles);
                    g.ho_div = make_fast_div(1);
                    lg.tile = tiles >= 4096 ? (o.cin % 128 == 0 ? T128x64k128 : T128x64) : (o.cin % 128 == 0 ? T64x64k128 : T64x64);
                    g.split_k = 1;
                    g.ktiles_per_split = g.K / conv_bk(g, false, lg.tile);
                    g.nz = 16;
                    g.zs_x = (long long)tiles * o.cin * esz;
                    g.zs_w = (long long)o.cout * o.cin * esz;
                    g.zs_y = (long long)tiles * o.cout * esz;
                    lg.x = Ref{SP_WORKSPACE, tmp_off[0]};
                    lg.w = Ref{SP_WEIGHTS, ws.wino_w_off};
                    lg.y = Ref{SP_WORKSPACE, tmp_off[1]};
                    const TileDim tdg = conv_tile_dim(lg.tile);
                    lg.info.gemm_m = tiles; lg.info.gemm_n = o.cout; lg.info.gemm_k = o.cin;
                    lg.info.flops = 2 * 16 * tiles * o.cout * o.cin;
                    lg.info.bytes = (int64_t)tmp_bytes[0] + (int64_t)ws.wino_bytes + (int64_t)tmp_bytes[1];
                    lg.info.tile_m = tdg.bm; lg.info.tile_n = tdg.bn; lg.info.tile_k = conv_bk(g, false, lg.tile); lg.info.split_k = 1;
                    lg.info.conv_tile = lg.tile; lg.info.wave_groups = tdg.kg;
                    snprintf(lg.info.name, sizeof lg.info.name, "winograd_16gemms");
                    p.launches.push_back(lg);
                    Launch lo{};
                    lo.kind = K_WINO_OUTPUT;
                    lo.op_index = i;
                    lo.wino = WinoArgs{nullptr, nullptr, nullptr, nullptr, batch, os.h, os.w, o.cout, th, tw, 0, o.relu};
                    lo.x = Ref{SP_WORKSPACE, tmp_off[1]};
                    lo.y = p.op_out[i];
                    lo.bias = Ref{SP_WEIGHTS, ws.packed_b_off};
                    if (o.residual_from >= 0) lo.res = p.op_out[o.residual_from];
                    const int64_t out_bw = (int64_t)batch * os.h * os.w * os.c * esz;
                    lo.info.bytes = (int64_t)tmp_bytes[1] + out_bw + (o.residual_from >= 0 ? out_bw : 0) + o.cout * 4;
                    snprintf(lo.info.name, sizeof lo.info.name, "winograd_output");
                    p.launches.push_back(lo);
                    break;
                }
                Launch l{};
                l.kind = K_CONV;
                l.op_index = i;
                l.stem = (i == 0);
                ConvArgs &a = l.conv;
                a.B = batch; a.H = sh; a.W = sw; a.Cin = ws.cinp; a.Ho = os.h; a.Wo = os.w; a.Cout = o.cout;
                a.kh = o.kh; a.kw = o.kw; a.kwp = ws.kwp; a.khp = ws.khp; a.stride = o.stride;
                conv_set_pad(a, o.pad, o.kh == o.kw ? o.pad : o.pad_w);
                conv_set_ld(a, o.input_from < 0 ? ws.cinp : p.op_ld[o.input_from], p.op_ld[i]);
                if (o.input_from < 0) { a.H = in_hp; a.W = in_wp; a.pad = 0; }  // the cast already padded the image
                a.M = batch * os.h * os.w;
                a.K = ws.khp * ws.kwp * ws.cinp;
                a.relu = o.relu;
                a.wo_div = make_fast_div((uint32_t)os.w);
                a.ho_div = make_fast_div((uint32_t)os.h);
                pick_conv_tile(a.M, a.Cout, (int64_t)o.kh * o.kw * o.cin, o.kh, o.stride, a.K / conv_bk(a, l.stem, T64x64), ov,
                               &l.tile, &a.split_k);
                if (l.stem) l.tile = conv_tile_one_group(l.tile);   // the first convolution's mode has no wave groups
                if (!conv_uses_dlds(a, l.stem)) l.tile = conv_tile_staged(l.tile);   // the register-staged kernel's shapes
                if (conv_bk(a, l.stem, l.tile) != conv_tile_dim(l.tile).bk) l.tile = conv_tile_k64(l.tile);  // Cin % 128 != 0
                const int ktiles = a.K / conv_bk(a, l.stem, l.tile);
                a.split_k = std::max(1, std::min(a.split_k, ktiles));
                {
                    const TileDim tdc = conv_tile_dim(l.tile);
                    const int64_t tiles = ((int64_t)a.M + tdc.bm - 1) / tdc.bm * ((a.Cout + tdc.bn - 1) / tdc.bn);
                    if (tiles * 4 > (int64_t)kCounterBytes || (int64_t)a.M * a.Cout * 4 >= (1ll << 31)) a.split_k = 1;
                }
                a.ktiles_per_split = (ktiles + a.split_k - 1) / a.split_k;
                a.split_k = (ktiles + a.ktiles_per_split - 1) / a.ktiles_per_split;  // no empty splits
                l.x = src;
                l.w = Ref{SP_WEIGHTS, ws.packed_w_off};
                l.bias = Ref{SP_WEIGHTS, ws.packed_b_off};
                l.y = p.op_out[i];
                if (o.residual_from >= 0) l.res = p.op_out[o.residual_from];
                const int64_t in_pixels = (o.kh == 1 && o.stride > 1) ? (int64_t)a.M : (int64_t)batch * sh * sw;
                const int64_t real_k = (int64_t)o.kh * o.kw * o.cin;
                const int64_t in_b = in_pixels * (i == 0 ? 4 : o.cin) * esz;
                const int64_t w_b = (int64_t)o.cout * real_k * esz + o.cout * 4;
                const int64_t out_b = (int64_t)batch * os.h * os.w * os.c * esz;
                const int64_t res_b = o.residual_from >= 0 ? out_b : 0;
                l.info.gemm_m = a.M; l.info.gemm_n = a.Cout; l.info.gemm_k = real_k;
                l.info.flops = 2 * (int64_t)a.M * a.Cout * real_k;
                const TileDim td = conv_tile_dim(l.tile);
                l.info.tile_m = td.bm; l.info.tile_n = td.bn; l.info.tile_k = conv_bk(a, l.stem, l.tile); l.info.split_k = a.split_k;
                l.info.conv_tile = l.tile; l.info.wave_groups = td.kg;
                a.panel_log2 = (ov.panels && !l.stem && conv_uses_dlds(a, false)) ? choose_panel(a.Cout, td.bn, w_b, in_b) : 0;
                l.info.panels = 1 << a.panel_log2;
                if (a.split_k > 1) {
                    partial_bytes = (size_t)a.split_k * a.M * a.Cout * 4;
                    partial_off = ws_alloc(partial_bytes);
                    l.partial = Ref{SP_WORKSPACE, partial_off};
                    l.counters = Ref{SP_WORKSPACE, 0};
                    // partial sums are written once and read once by the tile's last workgroup
                    l.info.bytes = in_b + w_b + out_b + res_b + 2 * (int64_t)partial_bytes;
                    snprintf(l.info.name, sizeof l.info.name, "conv%dx%d_s%d_splitk%d", o.kh, o.kw, o.stride, a.split_k);
                } else {
                    l.info.bytes = in_b + w_b + out_b + res_b;
                    l.in_bytes = in_b;
                    snprintf(l.info.name, sizeof l.info.name, i == 0 ? "stem%dx%d_s%d" : "conv%dx%d_s%d", o.kh, o.kw, o.stride);
                }
                p.launches.push_back(l);
                break;
            }
            case CW_OP_CONCAT: {
                place_output(i, (size_t)batch * os.h * os.w * os.c * esz);
                const int srcs[2] = {o.input_from, o.residual_from};
                const int at[2] = {0, m.shapes[o.input_from].c};
                for (int k = 0; k < 2; ++k) {
                    const int sidx = srcs[k];
                    if (host[sidx] == i && !(k == 1 && sidx == srcs[0])) continue;   // it wrote its channels itself
                    Launch l{};
                    l.kind = K_COPY_CHANNELS;
                    l.op_index = i;
                    l.copy = CopyArgs{nullptr, nullptr, batch * os.h * os.w, m.shapes[sidx].c, p.op_ld[sidx], p.op_ld[i]};
                    l.x = p.op_out[sidx];
                    l.y = Ref{SP_WORKSPACE, p.op_out[i].offset + (size_t)at[k] * esz};
                    l.info.bytes = 2 * (int64_t)batch * os.h * os.w * m.shapes[sidx].c * esz;
                    snprintf(l.info.name, sizeof l.info.name, "concat_copy");
                    p.launches.push_back(l);
                }
                break;
            }
            case CW_OP_MAXPOOL: {
                out_bytes[i] = (size_t)batch * os.h * os.w * os.c * esz;
                p.op_out[i] = Ref{SP_WORKSPACE, ws_alloc(out_bytes[i])};
                Launch l{};
                l.kind = K_MAXPOOL;
                l.op_index = i;
                l.pool = PoolArgs{nullptr, nullptr, batch, sh, sw, sc, os.h, os.w, o.kh, o.stride, o.pad};
                l.x = src; l.y = p.op_out[i];
                l.info.bytes = (int64_t)batch * sh * sw * sc * esz + (int64_t)out_bytes[i];
                snprintf(l.info.name, sizeof l.info.name, "maxpool%dx%d_s%d", o.kh, o.kw, o.stride);
                if (pool_conv[i] >= 0) {
                    const int k = pool_conv[i];
                    const cw_op &oc = m.ops[k];
                    const WeightSlot &wsc = m.wslots[m.op_wslot[k]];
                    out_bytes[k] = (size_t)batch * os.h * os.w * oc.cout * esz;
                    p.op_out[k] = Ref{SP_WORKSPACE, ws_alloc(out_bytes[k])};
                    p.op_ld[k] = oc.cout;
                    l.pool_bm = pool_bm[i];
                    ConvArgs &a = l.conv;
                    a.B = batch; a.H = os.h; a.W = os.w; a.Cin = oc.cin; a.Ho = os.h; a.Wo = os.w; a.Cout = oc.cout;
                    a.kh = 1; a.kw = 1; a.kwp = 1; a.khp = 1; a.stride = 1;
                    conv_set_pad(a, 0, 0);
                    conv_set_ld(a, oc.cin, oc.cout);
                    a.M = batch * os.h * os.w;
                    a.K = oc.cin;
                    a.relu = oc.relu;
                    a.split_k = 1; a.ktiles_per_split = 1;
                    l.w = Ref{SP_WEIGHTS, wsc.packed_w_off};
                    l.bias = Ref{SP_WEIGHTS, wsc.packed_b_off};
                    l.y2 = p.op_out[k];
                    l.info.fused_op = k;
                    l.info.gemm_m = a.M; l.info.gemm_n = a.Cout; l.info.gemm_k = a.K;
                    l.info.flops = 2 * (int64_t)a.M * a.Cout * a.K;
                    l.info.bytes += (int64_t)oc.cout * oc.cin * esz + oc.cout * 4 + (int64_t)out_bytes[k];   // its input never leaves the chip
                    const size_t len = strlen(l.info.name);
                    snprintf(l.info.name + len, sizeof l.info.name - len, "+1x1");
                }
                p.launches.push_back(l);
                break;
            }
            case CW_OP_GAVGPOOL: {
                out_bytes[i] = (size_t)batch * os.c * 4;
                p.op_out[i] = Ref{SP_WORKSPACE, ws_alloc(out_bytes[i])};
                Launch l{};
                l.kind = K_GAVGPOOL;
                l.op_index = i;
                l.pool = PoolArgs{nullptr, nullptr, batch, sh, sw, sc, 1, 1, 0, 1, 0};
                l.x = src; l.y = p.op_out[i];
                l.info.bytes = (int64_t)batch * sh * sw * sc * esz + (int64_t)out_bytes[i];
                snprintf(l.info.name, sizeof l.info.name, "global_avgpool");
                p.launches.push_back(l);
                break;
            }
            case CW_OP_FC: {
                const WeightSlot &ws = m.wslots[m.op_wslot[i]];
                p.op_out[i] = Ref{SP_SLOT_LOGITS, 0};
                Launch l{};
                l.kind = K_FC;
                l.op_index = i;
                l.fc.B = batch; l.fc.In = o.cin; l.fc.Out = o.cout;
                l.x = src;
                l.w = Ref{SP_WEIGHTS, ws.packed_w_off};
                l.bias = Ref{SP_WEIGHTS, ws.packed_b_off};
                l.y = p.op_out[i];
                l.info.gemm_m = batch; l.info.gemm_n = o.cout; l.info.gemm_k = o.cin;
                l.info.flops = 2 * (int64_t)batch * o.cout * o.cin;
                l.info.bytes = (int64_t)batch * o.cin * 4 + (int64_t)o.cout * o.cin * esz + o.cout * 4 + (int64_t)batch * o.cout * 4;
                snprintf(l.info.name, sizeof l.info.name, "fc");
                // The softmax that follows (model_init has checked that it does) runs in the same
                // launch where the finishing workgroup can hold every row in registers.
                if (ov.fc_softmax && batch <= kFcSoftmaxMaxBatch && o.cout <= kFcSoftmaxMaxOut) {
                    l.fc.split_k = o.cin % 512 == 0 ? 4 : 2;   // cin % 256 == 0 holds for every FC
                    partial_bytes = (size_t)l.fc.split_k * 16 * o.cout * 4;
                    partial_off = ws_alloc(partial_bytes);
                    l.partial = Ref{SP_WORKSPACE, partial_off};
                    l.counters = Ref{SP_WORKSPACE, 0};
                    l.probs = Ref{SP_SLOT_PROBS, 0};
                    l.info.split_k = l.fc.split_k;
                }
                p.launches.push_back(l);
                break;
            }
            case CW_OP_SOFTMAX: {
                p.op_out[i] = Ref{SP_SLOT_PROBS, 0};
                if (!p.launches.empty() && p.launches.back().kind == K_FC && p.launches.back().probs.space == SP_SLOT_PROBS) {
                    Launch &lf = p.launches.back();   // computed by the FC's launch
                    lf.info.fused_op = lf.op_index;
                    lf.op_index = i;
                    lf.info.bytes += (int64_t)batch * o.cout * 4;   // the probabilities; the logits are not read back from HBM
                    snprintf(lf.info.name, sizeof lf.info.name, "fc+softmax");
                    break;
                }
                Launch l{};
                l.kind = K_SOFTMAX;
                l.op_index = i;
                l.sm.B = batch; l.sm.D = o.cout;
                l.x = src; l.y = p.op_out[i];
                l.info.bytes = 2 * (int64_t)batch * o.cout * 4;
                snprintf(l.info.name, sizeof l.info.name, "softmax");
                p.launches.push_back(l);
                break;
            }
        }

        if (partial_bytes) arena.free(partial_off, partial_bytes);
        for (int k = 0; k < 2; ++k)
            if (tmp_bytes[k]) arena.free(tmp_off[k], tmp_bytes[k]);
        if (!no_reuse) {
            if (i == 0) arena.free(cast_off, cast_bytes);
            for (int j = 0; j < n_ops; ++j) {
                if (pos[j] > t) continue;
                const bool dead_now = (last_use[j] == t) || (j == i && last_use[j] < 0);
                if (dead_now && p.op_out[j].space == SP_WORKSPACE && out_bytes[j]) {
                    arena.free(p.op_out[j].offset, out_bytes[j]);
                    out_bytes[j] = 0;
                }
            }
        }
    }

    // Two consecutive convolution launches that read the same tensor and do not depend on each other
    // (in a ResNet: the first 1x1 of a block and the projection shortcut beside it) become one
    // launch on one tile shape: that of the one with more work, if the pair kernel has it and the
    // other is at least a tile wide.
    if (ov.pair && !resident && ov.tile < 0 && ov.split_k <= 0) {
        for (size_t i = 0; i + 1 < p.launches.size(); ++i) {
            Launch &l0 = p.launches[i], &l1 = p.launches[i + 1];
            if (l0.kind != K_CONV || l1.kind != K_CONV || l0.stem || l1.stem || l0.fused_bm > 0 || l1.fused_bm > 0) continue;
            if (l0.pair_op >= 0 || l1.pair_op >= 0 || l0.conv.split_k != 1 || l1.conv.split_k != 1) continue;
            if (l0.x.space != l1.x.space || l0.x.offset != l1.x.offset || l0.conv.Cin != l1.conv.Cin || l0.conv.Cin % 64 != 0) continue;
            if (m.ops[l1.op_index].input_from == l0.op_index || m.ops[l1.op_index].residual_from == l0.op_index) continue;
            const ConvTile cand[2] = {l1.info.flops >= l0.info.flops ? l1.tile : l0.tile, l1.info.flops >= l0.info.flops ? l0.tile : l1.tile};
            int pick = -1;
            for (int k = 0; k < 2 && pick < 0; ++k) {
                const TileDim d = conv_tile_dim(cand[k]);
                if (conv_pair_tile_ok(cand[k]) && l0.conv.Cin % d.bk == 0 && d.bn <= l0.conv.Cout && d.bn <= l1.conv.Cout) pick = k;
            }
            if (pick < 0) continue;
            const ConvTile tile = cand[pick];
            const TileDim d = conv_tile_dim(tile);
            Launch l = l1;
            l.tile = tile;
            l.pair_op = l0.op_index;
            l.conv0 = l0.conv;
            l.conv0.ktiles_per_split = l.conv0.K / d.bk;
            l.conv.ktiles_per_split = l.conv.K / d.bk;
            // both members run on the pair's tile shape: their tile numbering is chosen for it
            l.conv0.panel_log2 = ov.panels ? choose_panel(l.conv0.Cout, d.bn, (int64_t)l.conv0.Cout * l.conv0.K * 2, l0.in_bytes) : 0;
            l.conv.panel_log2 = ov.panels ? choose_panel(l.conv.Cout, d.bn, (int64_t)l.conv.Cout * l.conv.K * 2, l1.in_bytes) : 0;
            l.info.panels = (1 << l.conv.panel_log2) | ((1 << l.conv0.panel_log2) << 8);
            l.w0 = l0.w; l.bias0 = l0.bias; l.res0 = l0.res; l.y0 = l0.y;
            l.info.flops = l0.info.flops + l1.info.flops;
            l.info.bytes = l0.info.bytes + l1.info.bytes - std::min(l0.in_bytes, l1.in_bytes);   // the shared input once
            l.info.tile_m = d.bm; l.info.tile_n = d.bn; l.info.tile_k = d.bk; l.info.conv_tile = tile; l.info.wave_groups = d.kg;
            char name[48];
            snprintf(name, sizeof name, "%.20s|%.20s", l0.info.name, l1.info.name);
            memcpy(l.info.name, name, sizeof l.info.name);
            p.launches[i] = l;
            p.launches.erase(p.launches.begin() + i + 1);
        }
    }
    // Resident runs: every maximal run of two or more plain convolution launches (direct-to-LDS
    // kernel, whole K per workgroup) becomes one launch whose members keep partition 0's arguments.
    if (res_mode) {
        constexpr int kResidentLateM = 4096;
        auto eligible = [&](const Launch &l) {
            return l.kind == K_CONV && !l.stem && l.fused_bm == 0 && l.pair_op < 0 && l.conv.nz <= 1 && l.conv.Cin % 64 == 0 &&
                   l.conv.kwp == l.conv.kw && l.conv.khp == l.conv.kh && (res_mode == 1 || l.conv.M <= kResidentLateM);
        };
        std::vector<Launch> out;
        for (size_t i = 0; i < p.launches.size();) {
            size_t j = i;
            while (j < p.launches.size() && eligible(p.launches[j])) ++j;
            if (j - i < 2) {
                for (size_t k = i; k < std::max(j, i + 1); ++k) out.push_back(p.launches[k]);
                i = std::max(j, i + 1);
                continue;
            }
            Launch r{};
            r.kind = K_RESIDENT;
            r.op_index = p.launches[j - 1].op_index;
            std::vector<int> member_of(n_ops, -1);
            int flag_base = 0;
            for (size_t k = i; k < j; ++k) {
                Launch mlaunch = p.launches[k];
                const cw_op &o = m.ops[mlaunch.op_index];
                ConvArgs &a = mlaunch.conv;
                a.B = batch / kResPartitions;
                a.M = a.B * a.Ho * a.Wo;
                const int v = pick_res_variant(a.M, a.Cout, a.K, a.Cin);
                const ResVariantDim d = res_variant_dim(v);
                a.split_k = 1;
                a.ktiles_per_split = a.K / d.bk;
                mlaunch.partial = Ref{};
                mlaunch.counters = Ref{};
                mlaunch.res_variant = v;
                mlaunch.res_tiles = ((a.M + d.bm - 1) / d.bm) * ((a.Cout + d.bn - 1) / d.bn);
                mlaunch.res_ps_x = (long long)a.B * a.H * a.W * conv_ldx(a) * (long long)esz;
                mlaunch.res_ps_y = (long long)a.M * conv_ldy(a) * (long long)esz;
                mlaunch.res_ps_res = (long long)a.M * a.Cout * (long long)esz;
                mlaunch.res_dep[0] = o.input_from >= 0 ? member_of[o.input_from] : -1;
                mlaunch.res_dep[1] = o.residual_from >= 0 ? member_of[o.residual_from] : -1;
                mlaunch.res_flag_base = flag_base;
                flag_base += mlaunch.res_tiles;
                mlaunch.info.tile_m = d.bm; mlaunch.info.tile_n = d.bn; mlaunch.info.tile_k = d.bk; mlaunch.info.split_k = 1;
                member_of[mlaunch.op_index] = (int)r.members.size();
                r.info.flops += mlaunch.info.flops;
                r.info.bytes += (int64_t)a.M * kResPartitions * 0 + mlaunch.info.bytes;
                r.members.push_back(mlaunch);
            }
            r.res_flags_per_part = flag_base;
            if ((size_t)kResPartitions * flag_base * 4 > kResidentBytes - kResidentFlagsOff)
                return fail(err, CW_ERR_NO_MEMORY, "batch %d: a resident run needs more completion flags than the workspace header holds", batch);
            // split-K members counted their partial sums; a resident member walks the whole K itself
            r.info.bytes = 0;
            for (const Launch &ml : r.members) {
                const cw_op &o = m.ops[ml.op_index];
                const ConvArgs &a = ml.conv;
                const int64_t Mfull = (int64_t)a.M * kResPartitions;
                const int64_t in_pixels = (o.kh == 1 && o.stride > 1) ? Mfull : (int64_t)batch * a.H * a.W;
                r.info.bytes += in_pixels * o.cin * (int64_t)esz + (int64_t)o.cout * a.K * (int64_t)esz + o.cout * 4 + Mfull * o.cout * (int64_t)esz * (o.residual_from >= 0 ? 2 : 1);
            }
            snprintf(r.info.name, sizeof r.info.name, "resident_%dconvs", (int)r.members.size());
            out.push_back(r);
            i = j;
        }
        p.launches.swap(out);
    }
    // grid/block of every launch, for introspection
    for (Launch &l : p.launches) {
        dim3 g(1, 1, 1);
        int b = 0;
        switch (l.kind) {
            case K_CONV:
                if (l.fused_bm > 0) conv_fused_grid(l.fused_bm, l.fused_kg, l.conv, &g, &b);
                else if (l.pair_op >= 0) conv_pair_grid(l.tile, l.conv0, l.conv, &g, &b);
                else conv_grid(l.tile, l.conv, &g, &b);
                break;
            case K_CAST_INPUT: g = dim3((unsigned)(((size_t)l.cast.B * l.cast.Hp * l.cast.Wp + 255) / 256)); b = 256; break;
            case K_MAXPOOL:
                if (l.pool_bm > 0) g = dim3((unsigned)(((size_t)l.pool.B * l.pool.Ho * l.pool.Wo + l.pool_bm - 1) / l.pool_bm));
                else g = dim3((unsigned)(((size_t)l.pool.B * l.pool.Ho * l.pool.Wo * (l.pool.C / 8) + 255) / 256));
                b = 256;
                break;
            case K_GAVGPOOL: g = dim3((unsigned)(l.pool.B * (l.pool.C / 64))); b = l.pool.H * l.pool.W >= kGapWideFrom ? 1024 : 64; break;
            case K_FC:
                if (l.probs.space == SP_SLOT_PROBS) { g = dim3((l.fc.Out + 15) / 16, l.fc.split_k); b = 256; }
                else { g = dim3((l.fc.Out + 15) / 16, (l.fc.B + 15) / 16); b = 512; }
                break;
            case K_SOFTMAX: g = dim3(l.sm.B); b = 256; break;
            case K_DWCONV:
                if (l.dw_fused) {
                    const long long M = (long long)l.dw.B * l.dw.Ho * l.dw.Wo;
                    const int bm = dwconv_conv_bm(l.dw.C, M);
                    g = dim3((unsigned)((M + bm - 1) / bm));
                }
                else g = dim3((unsigned)(((size_t)l.dw.B * l.dw.Ho * l.dw.Wo * (l.dw.C / 8) + 255) / 256));
                b = 256;
                break;
            case K_COPY_CHANNELS: g = dim3((unsigned)(((size_t)l.copy.pixels * (l.copy.C / 8) + 255) / 256)); b = 256; break;
            case K_RESIDENT: g = dim3(kResPartitions * kResGroupsPerPartition); b = 256; break;
            case K_WINO_INPUT:
            case K_WINO_OUTPUT: g = dim3((unsigned)(((size_t)l.wino.B * l.wino.th * l.wino.tw * (l.wino.C / 8) + 255) / 256)); b = 256; break;
        }
        l.info.op_index = l.op_index;
        const bool fc_sm = l.kind == K_FC && l.probs.space == SP_SLOT_PROBS;   // fused_op = the FC, set where the softmax joined it
        const bool pool_conv1x1 = l.kind == K_MAXPOOL && l.pool_bm > 0;       // fused_op = the 1x1 convolution over the pooled tile
        if (l.fused_bm <= 0) { if (!fc_sm && !pool_conv1x1 && !l.dw_fused) l.info.fused_op = -1; l.info.proj_op = -1; l.info.next_op = -1; }
        l.info.pair_op = l.pair_op;
        l.info.kind = l.kind;
        if (l.kind != K_CONV) { l.info.conv_tile = -1; l.info.wave_groups = 1; }
        l.info.grid_x = g.x; l.info.grid_y = g.y; l.info.grid_z = g.z; l.info.block = b;
        if (l.info.split_k == 0) l.info.split_k = 1;
    }
    p.workspace_bytes = arena.high_water();
    *out = std::move(p);
    return CW_OK;
}

}  // namespace cw
