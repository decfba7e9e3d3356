"""The C-ABI library loads, exports every symbol the header declares, and its host
logic (model validation, plan compiler, allocator behaviour) works without a GPU."""
import os
import re

import numpy as np
import pytest

import paper_2006_02464_amd as cw
from oracle import topology as T
from workload import gen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for h in sorted(os.listdir(inc)):
        if not h.endswith(".h"):
            continue
        text = open(os.path.join(inc, h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(cw_[a-z_0-9]+)\s*\(", text))
    return names


def test_every_declared_symbol_is_exported_and_bound():
    names = _header_symbols()
    assert len(names) >= 34
    lib = cw.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert names == set(cw.SIGNATURES), names ^ set(cw.SIGNATURES)


def test_strerror():
    lib = cw.lib()
    assert lib.cw_strerror(0) == b"ok"
    seen = {lib.cw_strerror(-i) for i in range(1, 13)}
    assert len(seen) == 12 and b"unknown status" not in seen
    assert lib.cw_strerror(-99) == b"unknown status"


@pytest.fixture()
def ctx():
    c = cw.Context(device=-1)        # planning-only context: no GPU touched
    yield c
    c.destroy()


@pytest.mark.parametrize("depth,hw", [(18, 64), (50, 224), (152, 224)])
def test_resnet_op_lists_match_the_oracle_topology(ctx, depth, hw):
    m = ctx.model_define_resnet(depth, hw, hw)
    ours = ctx.model_get_ops(m)
    ref = [tuple(o) for o in T.resnet(depth)]
    assert ours == ref
    assert ctx.model_weight_bytes(m) == gen.blob_bytes(T.weight_shapes(T.resnet(depth)))


def test_resnet_plans_fit_the_static_arena(ctx):
    """cw_exec_static keeps a plan's intermediates in an array built into the library: the plans of
    the metric's models must fit it at every batch size."""
    from paper_2006_02464_amd import binding
    cap = binding.lib().cw_exec_static_capacity()
    for depth, dtype in ((50, "fp16"), (152, "bf16")):
        m = ctx.model_define_resnet(depth, 224, 224, dtype)
        for b in (1, 2, 4, 8, 16):
            assert ctx.model_workspace_bytes(m, b) <= cap, (depth, b)


def test_plan_is_fixed_and_covers_every_op(ctx):
    m = ctx.model_define_resnet(50, 224, 224)
    m2 = ctx.model_define_resnet(50, 224, 224)
    for b in (1, 2, 4, 8, 16):
        plan = ctx.plan(m, b)
        assert plan == ctx.plan(m2, b)                      # pure function of (model, batch)
        ops_hit = ({l["op_index"] for l in plan} | {l["fused_op"] for l in plan if l["fused_op"] >= 0} |
                   {l["proj_op"] for l in plan if l["proj_op"] >= 0} | {l["pair_op"] for l in plan if l["pair_op"] >= 0} |
                   {l["next_op"] for l in plan if l["next_op"] >= 0})
        assert ops_hit == set(range(57))                    # a fused launch covers two or three ops, a pair launch two
        assert len(plan) == 58 - sum((l["fused_op"] >= 0) + (l["proj_op"] >= 0) + (l["pair_op"] >= 0) + (l["next_op"] >= 0) for l in plan)
        flops = sum(l["flops"] for l in plan)
        assert flops == 2 * b * T.mac_count(T.resnet(50), 224, 224)
        for l in plan:
            assert l["grid_x"] >= 1 and l["block"] in (64, 128, 256, 512, 1024)
            if l["name"].startswith("conv") and l["split_k"] == 1 and l["pair_op"] < 0:
                tiles = -(-l["gemm_m"] // l["tile_m"]) * -(-l["gemm_n"] // l["tile_n"])
                assert l["grid_x"] == tiles and l["grid_y"] == 1
        ws = ctx.model_workspace_bytes(m, b)
        assert 0 < ws <= 512 << 20
    assert ctx.model_workspace_bytes(m, 16) > ctx.model_workspace_bytes(m, 1)
    with pytest.raises(cw.CwError) as e:
        ctx.plan_num_launches(m, 3)
    assert e.value.status == cw.CW_ERR_BAD_BATCH


def test_debug_keep_uses_more_workspace(ctx):
    m = ctx.model_define_resnet(18, 64, 64)
    ctx.set_debug_keep(True)
    k = ctx.model_define_resnet(18, 64, 64)
    assert ctx.model_workspace_bytes(k, 16) > ctx.model_workspace_bytes(m, 16)


def test_plan_override_reaches_every_tile(ctx):
    for name, idx in cw.CONV_TILES.items():
        ctx.set_plan_override(idx, 2)
        m = ctx.model_define_resnet(18, 64, 64)
        bm, bn = (int(v) for v in re.sub(r"(w2|w8|k128|g2|g4|g8)", "", name).split("x"))
        convs = [l for l in ctx.plan(m, 4) if l["name"].startswith(("conv", "stem"))]
        assert convs and all((l["tile_m"], l["tile_n"]) == (bm, bn) for l in convs)
        ops = ctx.model_get_ops(m)
        for l in convs:
            cin = ops[l["op_index"]][1]
            # K slices: 64 for the first convolution (stride 2: two padded filter rows per slice),
            # 128 only where the tile asks and cin allows
            want = 64 if cin < 32 else (128 if "k128" in name and cin % 128 == 0 else 64)
            assert l["tile_k"] == want
            assert l["split_k"] == 2 or l["gemm_k"] <= l["tile_k"] or cin < 32   # one K slice cannot be split
    ctx.set_plan_override(-1, 0)


def _ops(*rows):
    return [tuple(r) for r in rows]


def test_model_validation_errors(ctx):
    C, MP, GAP, FC, SM = 0, 1, 2, 3, 4
    good = _ops((C, 3, 64, 7, 7, 2, 3, 1, -1, -1), (MP, 64, 64, 3, 3, 2, 1, 0, -1, 0),
                (C, 64, 512, 3, 3, 1, 1, 1, -1, 1), (GAP, 512, 512, 0, 0, 1, 0, 0, -1, 2),
                (FC, 512, 10, 1, 1, 1, 0, 0, -1, 3), (SM, 10, 10, 0, 0, 1, 0, 0, -1, 4))
    assert ctx.model_define(good, 3, 32, 32) >= 0

    def bad(ops, status, **kw):
        with pytest.raises(cw.CwError) as e:
            ctx.model_define(ops, kw.get("c", 3), 32, 32, dtype=kw.get("dtype", "fp16"))
        assert e.value.status == status, e.value

    bad(good[:-1], cw.CW_ERR_UNSUPPORTED)                                     # must end FC, SOFTMAX
    b = list(good); b[2] = (C, 64, 500, 3, 3, 1, 1, 1, -1, 1)                 # cout % 32
    bad(b, cw.CW_ERR_UNSUPPORTED)
    b = list(good); b[2] = (C, 32, 512, 3, 3, 1, 1, 1, -1, 1)                 # cin mismatch
    bad(b, cw.CW_ERR_INVALID)
    b = list(good); b[2] = (C, 64, 512, 3, 3, 1, 1, 1, 0, 1)                  # residual shape mismatch
    bad(b, cw.CW_ERR_INVALID)
    b = list(good); b[2] = (C, 64, 512, 3, 3, 1, 1, 1, -1, 2)                 # reads itself
    bad(b, cw.CW_ERR_INVALID)
    b = list(good); b[0] = (C, 8, 64, 7, 7, 2, 3, 1, -1, -1)                  # first conv cin > 4
    bad(b, cw.CW_ERR_UNSUPPORTED, c=8)
    b = list(good); b[0] = (C, 3, 64, 7, 5, 2, 3, 1, -1, -1)                  # non-square first conv
    bad(b, cw.CW_ERR_UNSUPPORTED)
    b = list(good); b[2] = (C, 64, 512, 3, 3, 1, 1, 3, -1, 1)                 # unknown activation code
    bad(b, cw.CW_ERR_UNSUPPORTED)
    b = list(good); b[2] = (C, 64, 512, 3, 3, 1, 1, 1, -1, 1, 0, 2)           # grouped but not depthwise
    bad(b, cw.CW_ERR_UNSUPPORTED)
    b = list(good); b[2] = (C, 64, 512, 7, 7, 1, 3, 1, -1, 1)                 # 49 taps
    bad(b, cw.CW_ERR_UNSUPPORTED)
    b = list(good); b[2] = (5, 64, 512, 0, 0, 1, 0, 0, 1, 1)                  # CONCAT whose channels do not add up
    bad(b, cw.CW_ERR_INVALID)
    ok = list(good); ok[2] = (C, 64, 512, 3, 5, 1, 1, 1, -1, 1, 2, 0)         # 3x5, padding (1, 2): same size out
    assert ctx.model_define(ok, 3, 32, 32) >= 0
    with pytest.raises(cw.CwError) as e:
        ctx.model_define(good, 3, 32, 32, batch_sizes=(0,))
    assert e.value.status == cw.CW_ERR_BAD_BATCH


def test_device_calls_on_planning_context_fail_loudly(ctx):
    m = ctx.model_define_resnet(18, 64, 64)
    blob = np.zeros(ctx.model_weight_bytes(m), np.uint8)
    with pytest.raises(cw.CwError):
        ctx.load_weights(m, blob)
    with pytest.raises(cw.CwError):
        ctx.input(m, 1, np.zeros((1, 3, 64, 64), np.float32))
    with pytest.raises(cw.CwError):
        ctx.exec(m, 1, 0)
    ctx.unload_weights(m)          # metadata only: always succeeds
    ctx.unload_weights(m)


def test_plan_table_rows_take_precedence(ctx):
    m0 = ctx.model_define_resnet(50, 224, 224)
    base = ctx.plan(m0, 16)
    target = next(l for l in base if l["kind"] == 1 and l["gemm_k"] == 2304 and l["fused_op"] < 0)   # a 3x3 of stage 3
    other = "64x32" if (target["tile_m"], target["tile_n"]) != (64, 32) else "32x64"
    ops = ctx.model_get_ops(m0)
    stride = ops[target["op_index"]][5]
    ctx.set_plan_table([(target["gemm_m"], target["gemm_n"], target["gemm_k"], 3, stride, other, 2)])
    try:
        m1 = ctx.model_define_resnet(50, 224, 224)
        plan = ctx.plan(m1, 16)
        for a, b in zip(base, plan):
            if a["kind"] == 1 and (a["gemm_m"], a["gemm_n"], a["gemm_k"], ops[a["op_index"]][5]) == (target["gemm_m"], target["gemm_n"], 2304, stride):
                assert "%dx%d" % (b["tile_m"], b["tile_n"]) == other and b["split_k"] == 2
            else:
                assert (a["tile_m"], a["tile_n"], a["split_k"]) == (b["tile_m"], b["tile_n"], b["split_k"])
        with pytest.raises(cw.CwError):
            ctx.set_plan_table([(1, 1, 1, 1, 1, 99, 1)])
    finally:
        ctx.set_plan_table([])
    m2 = ctx.model_define_resnet(50, 224, 224)
    assert ctx.plan(m2, 16) == base


def test_fusion_of_bottleneck_tail(ctx):
    """At batch 16 the 3x3 + 1x1 tail of every stage-1 and stage-2 bottleneck of ResNet-50 is one
    launch; with fusion off or at batch 1 (too few pixels) it is two.  Debug retention keeps the
    fused plan (so that the fused launches can be compared with the oracle layer by layer): only
    the intermediate tensor of a fused launch has no place to be read back from."""
    m = ctx.model_define_resnet(50, 224, 224)
    ops = ctx.model_get_ops(m)
    fused = [l for l in ctx.plan(m, 16) if l["fused_op"] >= 0 and l["kind"] == 1]
    assert len(fused) == 7
    assert [l["proj_op"] >= 0 for l in fused] == [True] + [False] * 6   # the stride-1 projection of the first block
    proj = ops[fused[0]["proj_op"]]
    assert proj[3] == 1 and proj[5] == 1 and proj[7] == 0 and proj[1] == 64 and proj[2] == 256
    for l in fused:
        first, second = ops[l["fused_op"]], ops[l["op_index"]]
        assert first[3] == 3 and second[3] == 1 and second[1] == first[2] and first[2] in (64, 128)
        assert l["grid_x"] == -(-l["gemm_m"] // l["tile_m"]) and l["grid_y"] == 1 and l["split_k"] == 1
    assert not [l for l in ctx.plan(m, 1) if l["fused_op"] >= 0 and l["kind"] == 1]
    # the next block's 1x1 reduce rides along, also in the launch that computes the first block's projection
    third = [l for l in fused if l["next_op"] >= 0]
    assert len(third) == 5 and [l["proj_op"] >= 0 for l in third] == [True] + [False] * 4
    for l in third:
        nxt, second, first = ops[l["next_op"]], ops[l["op_index"]], ops[l["fused_op"]]
        assert l["next_op"] == l["op_index"] + 1 and nxt[9] == l["op_index"] and nxt[3] == 1 and nxt[5] == 1
        assert nxt[1] == second[2] and nxt[2] == first[2] and l["name"].endswith("+1x1+proj+1x1" if l["proj_op"] >= 0 else "+1x1+1x1")
    assert not any(l["op_index"] in {t["next_op"] for t in third} for l in ctx.plan(m, 16))   # no launch of their own
    ctx.set_fusion_third(0)
    try:
        m4 = ctx.model_define_resnet(50, 224, 224)
        assert not [l for l in ctx.plan(m4, 16) if l["next_op"] >= 0]
        assert len(ctx.plan(m4, 16)) == len(ctx.plan(m, 16)) + 5
    finally:
        ctx.set_fusion_third(1)
    ctx.set_fusion(0)
    try:
        m2 = ctx.model_define_resnet(50, 224, 224)
        assert not [l for l in ctx.plan(m2, 16) if l["fused_op"] >= 0 and l["kind"] == 1]
    finally:
        ctx.set_fusion(1)
    ctx.set_debug_keep(True)
    try:
        m3 = ctx.model_define_resnet(50, 224, 224)
        kept = [l for l in ctx.plan(m3, 16) if l["fused_op"] >= 0 and l["kind"] == 1]
        assert [(l["fused_op"], l["op_index"], l["proj_op"]) for l in kept] == [
            (l["fused_op"], l["op_index"], l["proj_op"]) for l in fused]
    finally:
        ctx.set_debug_keep(False)


def test_max_pool_with_the_1x1_behind_it(ctx):
    """From batch 2 up the max pool of ResNet-50 also computes the first bottleneck's 1x1 reduce (64 -> 64
    over the pooled tile); at batch 1 (49 workgroups) and with the option or all fusion off they are two
    launches; ResNet-18's max pool is followed by a 3x3 and stays alone."""
    m = ctx.model_define_resnet(50, 224, 224)
    ops = ctx.model_get_ops(m)
    assert [len(ctx.plan(m, b)) for b in (1, 2, 4, 8, 16)] == [54, 48, 48, 41, 41]
    for b in (2, 4, 8, 16):
        plan = ctx.plan(m, b)
        pool = [l for l in plan if l["kind"] == 3]
        assert len(pool) == 1 and pool[0]["op_index"] == 1 and pool[0]["fused_op"] == 2 and pool[0]["name"] == "maxpool3x3_s2+1x1"
        assert ops[2][0] == 0 and ops[2][3] == 1 and ops[2][1] == 64 and ops[2][2] == 64 and ops[2][9] == 1
        assert pool[0]["grid_x"] == -(-b * 56 * 56 // 64) and pool[0]["block"] == 256
        assert (pool[0]["gemm_m"], pool[0]["gemm_n"], pool[0]["gemm_k"]) == (b * 56 * 56, 64, 64) and pool[0]["flops"] == 2 * b * 56 * 56 * 64 * 64
        assert not [l for l in plan if l["kind"] == 1 and l["op_index"] == 2]      # no launch of its own
    assert [l["fused_op"] for l in ctx.plan(m, 1) if l["kind"] == 3] == [-1]
    for setter in (ctx.set_fusion_pool, ctx.set_fusion):
        setter(0)
        try:
            m2 = ctx.model_define_resnet(50, 224, 224)
            assert [l["fused_op"] for l in ctx.plan(m2, 16) if l["kind"] == 3] == [-1]
            assert [l for l in ctx.plan(m2, 16) if l["kind"] == 1 and 2 in (l["op_index"], l["pair_op"])]   # a launch of its own, or half of a pair
        finally:
            setter(1)
    m18 = ctx.model_define_resnet(18, 224, 224)
    assert [l["fused_op"] for l in ctx.plan(m18, 16) if l["kind"] == 3] == [-1]


def test_depthwise_with_the_1x1_behind_it(ctx):
    """MobileNet's first two depthwise-separable blocks (32 and 64 channels) are one launch each where the launch has
    96 workgroups of 64 pixels; the 128-channel ones and everything behind them stay two launches."""
    from oracle import topology as T
    ops = [tuple(o) for o in T.mobilenet()]
    m = ctx.model_define(ops, 3, 224, 224)
    assert [len(ctx.plan(m, b)) for b in (1, 4, 16)] == [30, 29, 29]
    for b, n in ((1, 1), (4, 2), (16, 2)):
        plan = ctx.plan(m, b)
        both = [l for l in plan if l["kind"] == 7 and l["fused_op"] >= 0]
        assert len(both) == n
        for l in both:
            dw, pw = ops[l["fused_op"]], ops[l["op_index"]]
            assert l["fused_op"] == l["op_index"] - 1 and dw[11] == dw[1] == dw[2] and dw[3] == 3 and pw[3] == 1 and pw[1] == dw[2] and dw[2] in (32, 64)
            assert l["grid_x"] == -(-l["gemm_m"] // 64) and l["grid_x"] >= 96 and l["block"] == 256 and l["gemm_k"] == dw[2] and l["gemm_n"] == pw[2]
            assert l["flops"] == 2 * l["gemm_m"] * dw[2] * 9 + 2 * l["gemm_m"] * pw[2] * pw[1]
        hit = {l["op_index"] for l in plan} | {l["fused_op"] for l in plan if l["fused_op"] >= 0} | {l["pair_op"] for l in plan if l["pair_op"] >= 0}
        assert hit == set(range(len(ops)))
    ctx.set_fusion_dw(0)
    try:
        m2 = ctx.model_define(ops, 3, 224, 224)
        assert [len(ctx.plan(m2, b)) for b in (1, 4, 16)] == [31, 31, 31]
    finally:
        ctx.set_fusion_dw(1)


def test_weight_pages():
    """The weight pool is paged (paper section 5.1): page counts per model, the limits, the free count."""
    c = cw.Context(device=-1, weight_pool_bytes=1 << 30)          # default page: 16 MiB
    try:
        assert c.weight_pages_free() == 64 and c.weight_pool_free() == 1 << 30
        pages = {d: c.model_weight_pages(c.model_define_resnet(d, 224, 224)) for d in (18, 50, 152)}
        assert pages == {18: 2, 50: 4, 152: 8}
    finally:
        c.destroy()
    c = cw.Context(device=-1, weight_pool_bytes=100 << 20, weight_page_bytes=8 << 20)
    try:
        assert c.weight_pages_free() == 12                        # the pool's tail below a page is unused
        m = c.model_define_resnet(50, 224, 224)
        n = c.model_weight_pages(m)
        packed_at_least = c.model_weight_bytes(m)                 # packing only ever pads
        assert -(-packed_at_least // (8 << 20)) <= n <= 8         # 51 MB: 7 pages minimum, little lost at page ends
        assert c.model_weight_pages(c.model_define_resnet(50, 224, 224)) == n   # a pure function of the model
    finally:
        c.destroy()
    c = cw.Context(device=-1, weight_page_bytes=4 << 20)          # ResNet's largest tensor (4.7 MB) does not fit a page
    try:
        with pytest.raises(cw.CwError) as e:
            c.model_define_resnet(18, 64, 64)
        assert e.value.status == cw.CW_ERR_UNSUPPORTED
    finally:
        c.destroy()
    with pytest.raises(cw.CwError):
        cw.Context(device=-1, weight_page_bytes=1000)             # not a multiple of 256


def test_pair_launches(ctx):
    """The first 1x1 of a bottleneck and the projection shortcut beside it read the same tensor: one
    launch (three at batch 16, where the first block's projection is already inside a fused launch;
    four at batch 1), unless switched off."""
    m = ctx.model_define_resnet(50, 224, 224)
    ops = ctx.model_get_ops(m)
    for batch, want in ((16, 3), (1, 4)):
        pairs = [l for l in ctx.plan(m, batch) if l["pair_op"] >= 0]
        assert len(pairs) == want
        for l in pairs:
            a, b = ops[l["pair_op"]], ops[l["op_index"]]
            assert a[9] == b[9] and a[0] == b[0] == 0 and a[3] == b[3] == 1      # same input, both 1x1 convolutions
            assert l["split_k"] == 1 and l["grid_y"] == 1
            tiles = lambda o, s: -(-(s // (o[5] * o[5])) // l["tile_m"]) * -(-o[2] // l["tile_n"])
            assert "|" in l["name"]
        assert sum(l["flops"] for l in ctx.plan(m, batch)) == 2 * batch * T.mac_count(T.resnet(50), 224, 224)
    ctx.set_pair_launches(0)
    try:
        m2 = ctx.model_define_resnet(50, 224, 224)
        assert not [l for l in ctx.plan(m2, 16) if l["pair_op"] >= 0]
        assert len(ctx.plan(m2, 16)) == len(ctx.plan(m, 16)) + 3
    finally:
        ctx.set_pair_launches(1)
