"""GPU tests of the boundary's action semantics: residency, slots, errors, timing."""
import math

import numpy as np
import pytest
import torch

import paper_2006_02464_amd as cw
from gpu_common import Case
from oracle import topology as T

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def setup():
    from paper_2006_02464_amd.runner import Worker
    # 8 weight pages of 8 MiB; a ResNet-18 takes 4 of them
    w = Worker(workspace_bytes=64 << 20, io_bytes=32 << 20, weight_pool_bytes=64 << 20,
               load_staging_bytes=32 << 20, weight_page_bytes=8 << 20)
    case = Case(T.resnet(18), 64, seed=0, dist="uniform")
    yield w, case
    w.close()


def _status(fn, *a, **k):
    with pytest.raises(cw.CwError) as e:
        fn(*a, **k)
    return e.value.status


def test_exec_checks_weights_and_input(setup):
    w, case = setup
    ctx = w.ctx
    mid = ctx.model_define_resnet(18, 64, 64)
    x = torch.zeros((1, 3, 64, 64), dtype=torch.float32).pin_memory()
    slot = ctx.input(mid, 1, x, w.stream)
    assert _status(ctx.exec, mid, 1, slot, w.stream) == cw.CW_ERR_NOT_LOADED
    w.load(mid, case.blob)
    assert _status(ctx.exec, mid, 2, slot, w.stream) == cw.CW_ERR_BAD_BATCH     # slot holds batch 1
    assert _status(ctx.exec, mid, 3, slot, w.stream) == cw.CW_ERR_BAD_BATCH     # no plan
    assert _status(ctx.exec, mid, 1, 63, w.stream) == cw.CW_ERR_NO_INPUT
    probs = torch.empty((1, 1000), dtype=torch.float32).pin_memory()
    assert _status(ctx.output, slot, probs, None, w.stream) == cw.CW_ERR_NO_INPUT  # no EXEC yet
    ctx.exec(mid, 1, slot, w.stream)
    ctx.exec(mid, 1, slot, w.stream)       # EXEC may be repeated on a slot
    assert ctx.exec_duration_ns(slot) > 0
    ctx.output(slot, probs, None, w.stream)
    w.stream.synchronize()
    assert abs(float(probs.sum()) - 1) < 1e-5
    assert _status(ctx.exec, mid, 1, slot, w.stream) == cw.CW_ERR_NO_INPUT      # slot was released
    assert _status(ctx.load_weights, mid, np.zeros(5, np.uint8)) == cw.CW_ERR_INVALID
    assert _status(w.load, mid, case.blob) == cw.CW_ERR_ALREADY_LOADED
    ctx.unload_weights(mid)
    ctx.unload_weights(mid)                # always succeeds


def test_load_aborts_when_pool_is_full_and_unload_frees(setup):
    w, case = setup
    ctx = w.ctx
    free0 = ctx.weight_pool_free()
    a = ctx.model_define_resnet(18, 64, 64)
    b = ctx.model_define_resnet(18, 64, 64)
    c = ctx.model_define_resnet(18, 64, 64)
    w.load(a, case.blob)
    w.load(b, case.blob)                   # 2 x 4 pages fill the pool of 8
    assert ctx.model_weight_pages(a) == 4 and ctx.weight_pages_free() == 0
    assert ctx.weight_pool_free() < free0 - 2 * 23_000_000
    assert _status(w.load, c, case.blob) == cw.CW_ERR_NO_MEMORY
    ctx.unload_weights(a)
    w.load(c, case.blob)                   # room again
    x = case.images(0, 2)
    za = w.infer(b, x)[1]
    zc = w.infer(c, x)[1]
    assert np.array_equal(za, zc)          # same weights, different pool regions
    for m in (b, c):
        ctx.unload_weights(m)
    assert ctx.weight_pool_free() == free0


def test_load_takes_any_free_pages(setup):
    """Paper section 5.1: weights live in pages and a LOAD takes whichever are free.  Two one-page
    models around a four-page one are unloaded: the 4 free pages are {0, 5, 6, 7}, no 4 of them
    adjacent.  A second ResNet-18 must still LOAD into them and compute bit for bit what the copy in
    pages 1-4 computes."""
    w, case = setup
    ctx = w.ctx
    O = T.Op
    small_ops = [O(T.CONV, 3, 64, 7, 7, 2, 3, 1, -1, -1), O(T.MAXPOOL, 64, 64, 3, 3, 2, 1, 0, -1, 0),
                 O(T.CONV, 64, 512, 3, 3, 1, 1, 1, -1, 1), O(T.GAVGPOOL, 512, 512, 0, 0, 1, 0, 0, -1, 2),
                 O(T.FC, 512, 10, 1, 1, 1, 0, 0, -1, 3), O(T.SOFTMAX, 10, 10, 0, 0, 1, 0, 0, -1, 4)]
    small = Case(small_ops, 32, seed=3, dist="uniform")
    assert ctx.weight_pages_free() == 8
    s1 = ctx.model_define([tuple(o) for o in small_ops], 3, 32, 32)
    s2 = ctx.model_define([tuple(o) for o in small_ops], 3, 32, 32)
    a = ctx.model_define_resnet(18, 64, 64)
    b = ctx.model_define_resnet(18, 64, 64)
    assert ctx.model_weight_pages(s1) == 1
    w.load(s1, small.blob)                 # page 0
    w.load(a, case.blob)                   # pages 1-4
    w.load(s2, small.blob)                 # page 5
    assert ctx.weight_pages_free() == 2
    assert _status(w.load, b, case.blob) == cw.CW_ERR_NO_MEMORY
    ctx.unload_weights(s1)
    ctx.unload_weights(s2)
    assert ctx.weight_pages_free() == 4    # 0, 5, 6, 7
    w.load(b, case.blob)
    assert ctx.weight_pages_free() == 0
    x = case.images(0, 4)
    za = np.concatenate([w.infer(a, x[i:i + 2])[1] for i in (0, 2)])
    zb = np.concatenate([w.infer(b, x[i:i + 2])[1] for i in (0, 2)])
    assert np.array_equal(za, zb)
    ref = case.oracle(x)["logits"]
    assert (np.abs(zb - ref).max(axis=1) / np.abs(ref).max(axis=1)).max() <= 2e-2
    # the small model again, now into a page that a ResNet-18 just used
    ctx.unload_weights(a)
    w.load(s1, small.blob)
    xs = small.images(0, 2)
    zs = w.infer(s1, xs, classes=10)[1]
    rs = small.oracle(xs)["logits"]
    assert (np.abs(zs - rs).max(axis=1) / np.abs(rs).max(axis=1)).max() <= 2e-2
    for m in (b, s1):
        ctx.unload_weights(m)
    assert ctx.weight_pages_free() == 8


def test_io_cache_exhaustion_and_reuse(setup):
    w, case = setup
    ctx = w.ctx
    mid = ctx.model_define_resnet(18, 64, 64)
    x = torch.zeros((16, 3, 64, 64), dtype=torch.float32).pin_memory()
    slots = []
    with pytest.raises(cw.CwError) as e:
        for _ in range(100):
            slots.append(ctx.input(mid, 16, x, w.stream))
    assert e.value.status in (cw.CW_ERR_NO_MEMORY, cw.CW_ERR_NO_SLOT)
    assert len(slots) >= 4
    for s in slots:
        ctx.release(s)
    s = ctx.input(mid, 16, x, w.stream)
    ctx.release(s)
    w.stream.synchronize()


def test_second_exec_on_another_stream_is_busy(setup):
    w, case = setup
    ctx = w.ctx
    mid = ctx.model_define_resnet(18, 224, 224)
    w.load(mid, case.blob)
    x = torch.zeros((16, 3, 224, 224), dtype=torch.float32).pin_memory()
    slot = ctx.input(mid, 16, x, w.stream)
    other = torch.cuda.Stream()
    with torch.cuda.stream(w.stream):       # ~50 ms of spinning ahead of the EXEC on its stream
        torch.cuda._sleep(120_000_000)
    ctx.exec(mid, 16, slot, w.stream)
    st = None
    try:
        ctx.exec(mid, 16, slot, other)
    except cw.CwError as e:
        st = e.status
    assert st == cw.CW_ERR_BUSY
    w.stream.synchronize()
    ctx.exec(mid, 16, slot, other)          # idle now: allowed
    other.synchronize()
    ctx.release(slot)
    ctx.unload_weights(mid)


def test_profile_measure(setup):
    w, case = setup
    ctx = w.ctx
    mid = ctx.model_define_resnet(18, 64, 64)
    w.load(mid, case.blob)
    assert ctx.profile_get(mid, 4)["n"] == 0
    prof, samples = ctx.profile_measure(mid, 4, 300, want_samples=True)
    assert prof["n"] == 300 and len(samples) == 300
    assert 0 < prof["min_us"] <= prof["p50_us"] <= prof["p99_us"] <= prof["p999_us"] <= prof["max_us"]
    s = np.sort(samples)
    rank = lambda q: s[min(300, max(1, math.ceil(q * 300))) - 1]     # nearest rank
    assert prof["p50_us"] == rank(0.50) and prof["p99_us"] == rank(0.99) and prof["p999_us"] == rank(0.999)
    assert ctx.profile_get(mid, 4) == prof
    per_launch = None
    x = torch.zeros((4, 3, 64, 64), dtype=torch.float32).pin_memory()
    slot = ctx.input(mid, 4, x, w.stream)
    per_launch = ctx.exec_timed_launches(mid, 4, slot, w.stream)
    assert len(per_launch) == ctx.plan_num_launches(mid, 4) and (per_launch > 0).all()
    # a profile over the caller's own input: the slot stays the caller's and keeps its input
    over_slot = ctx.profile_measure(mid, 4, 64, slot=slot)
    assert over_slot["n"] == 64 and 0.5 * prof["p50_us"] < over_slot["p50_us"] < 2 * prof["p50_us"]
    assert _status(ctx.profile_measure, mid, 2, 8, slot=slot) == cw.CW_ERR_BAD_BATCH
    assert _status(ctx.profile_measure, mid, 4, 8, slot=40) == cw.CW_ERR_NO_INPUT
    ctx.exec(mid, 4, slot, w.stream)
    ctx.release(slot)
    ctx.unload_weights(mid)


def test_graph_replay_equals_plain_launches(setup):
    """EXEC through the recorded graph and EXEC as plain launches give bit-identical results,
    on every replay, with other work and synchronisations in between."""
    w, case = setup
    ctx = w.ctx
    mid = ctx.model_define_resnet(18, 64, 64)
    w.load(mid, case.blob)
    x = case.images(0, 4)
    ctx.set_use_graphs(False)
    plain = w.infer(mid, x)[1]
    ctx.set_use_graphs(True)
    for i in range(6):
        got = w.infer(mid, x)[1]
        assert np.array_equal(got, plain), "replay %d differs" % i
        ctx.set_use_graphs(False)                       # eager work between replays
        other = w.infer(mid, case.images(10 + i, 4))[1]
        ctx.set_use_graphs(True)
        assert not np.array_equal(other, plain)
        torch.cuda.synchronize()
    # a model loaded while graphs are off runs without one, and still agrees
    ctx.set_use_graphs(False)
    m2 = ctx.model_define_resnet(18, 64, 64)
    w.load(m2, case.blob)
    ctx.set_use_graphs(True)
    assert np.array_equal(w.infer(m2, x)[1], plain)
    ctx.unload_weights(mid)
    ctx.unload_weights(m2)


def test_load_in_steps(setup):
    """LOAD as the executors issue it: an EXEC between the begin and the end step runs plain
    launches, one after the end step replays the graphs; both give what a one-call LOAD gives.
    Graphs recorded for a placement the model has left meanwhile are dropped."""
    w, case = setup
    ctx = w.ctx
    x = case.images(0, 4)
    ref = ctx.model_define_resnet(18, 64, 64)
    w.load(ref, case.blob)
    want = w.infer(ref, x)[1]
    ctx.unload_weights(ref)
    mid = ctx.model_define_resnet(18, 64, 64)
    from paper_2006_02464_amd.runner import pinned_like
    blob = pinned_like(case.blob)
    pd = ctx.load_weights_begin(mid, blob, w.stream)
    assert np.array_equal(w.infer(mid, x)[1], want)
    ctx.load_weights_record(pd)
    assert np.array_equal(w.infer(mid, x)[1], want)
    ctx.load_weights_end(pd)
    ctx.load_weights_release(pd)
    for _ in range(3):
        assert np.array_equal(w.infer(mid, x)[1], want)
    # unloaded (and loaded elsewhere) between record and end: the recorded graphs must not be used
    ctx.unload_weights(mid)
    pd = ctx.load_weights_begin(mid, blob, w.stream)     # pages 0..3 again
    ctx.load_weights_record(pd)
    ctx.unload_weights(mid)
    w.load(ref, case.blob)                               # takes pages 0..3
    w.load(mid, case.blob)                               # pages 4..7
    ctx.load_weights_end(pd)
    ctx.load_weights_release(pd)
    assert np.array_equal(w.infer(mid, x)[1], want)
    assert np.array_equal(w.infer(ref, x)[1], want)
    ctx.unload_weights(mid)
    ctx.unload_weights(ref)


def test_unload_then_load_waits_for_the_exec_in_flight(setup):
    """UNLOAD hands the pages back at once; a LOAD of another model on another stream takes them
    while EXECs of the unloaded model are still queued.  Those EXECs must read intact weights: the
    LOAD's pack kernels wait for the last EXEC that reads the pages."""
    from gpu_common import TOL, rel_err_per_sample
    w, case = setup
    ctx = w.ctx
    a = ctx.model_define_resnet(18, 64, 64)
    b = ctx.model_define_resnet(18, 64, 64)
    other = Case(T.resnet(18), 64, seed=9, dist="uniform")
    w.load(a, case.blob)
    x = case.images(0, 16)
    ref = case.oracle(x)["logits"]
    hx = torch.from_numpy(x.copy()).pin_memory()
    blob_b = torch.from_numpy(other.blob.copy()).pin_memory()
    s2 = torch.cuda.Stream()
    slot = ctx.input(a, 16, hx, w.stream)
    for _ in range(40):                       # a few milliseconds of EXECs queued on stream 1
        ctx.exec(a, 16, slot, w.stream)
    pages_before = ctx.weight_pages_free()
    ctx.unload_weights(a)
    assert ctx.weight_pages_free() == pages_before + ctx.model_weight_pages(a)
    ctx.load_weights(b, blob_b, s2)           # lowest free pages first: the ones A just gave back
    probs = torch.empty((16, 1000), dtype=torch.float32).pin_memory()
    logits = torch.empty((16, 1000), dtype=torch.float32).pin_memory()
    ctx.output(slot, probs, logits, w.stream)
    w.stream.synchronize()
    s2.synchronize()
    assert rel_err_per_sample(logits.numpy(), ref).max() <= TOL
    # and B is what was loaded: its own logits against the oracle
    xb = other.images(0, 2)
    got = w.infer(b, xb)[1]
    assert rel_err_per_sample(got, other.oracle(xb)["logits"]).max() <= TOL
    ctx.unload_weights(b)


def test_graph_recorded_for_other_pages_is_not_replayed(setup):
    """LOAD with graphs on (pages P), graphs off, UNLOAD, LOAD into other pages (no recording),
    graphs on again: EXEC must not replay the graph that holds the addresses of P."""
    from gpu_common import TOL, rel_err_per_sample
    w, case = setup
    ctx = w.ctx
    a = ctx.model_define_resnet(18, 64, 64)
    filler = ctx.model_define_resnet(18, 64, 64)
    x = case.images(0, 2)
    ref = case.oracle(x)["logits"]
    w.load(a, case.blob)                      # graphs recorded for the lowest pages
    first = w.infer(a, x)[1]
    ctx.unload_weights(a)
    try:
        ctx.set_use_graphs(0)
        w.load(filler, Case(T.resnet(18), 64, seed=4, dist="uniform").blob)   # takes A's old pages
        w.load(a, case.blob)                  # lands in other pages; nothing is recorded
    finally:
        ctx.set_use_graphs(1)
    got = w.infer(a, x)[1]
    assert rel_err_per_sample(got, ref).max() <= TOL
    assert np.array_equal(got, first)
    ctx.unload_weights(a)
    ctx.unload_weights(filler)
