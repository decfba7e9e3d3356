"""The worker's executors (paper section 5.2): actions with earliest / latest, one result each.
The window logic runs without a GPU on a planning-only context (UNLOAD is metadata only; LOAD and
INFER come back with the error of their first device call); the GPU test runs real actions."""
import time

import numpy as np
import pytest

import paper_2006_02464_amd as cw
from paper_2006_02464_amd.binding import CW_ACTION_INFER, CW_ACTION_LOAD, CW_ACTION_UNLOAD, Executors

MS = 1_000_000


@pytest.fixture()
def planning():
    ctx = cw.Context(device=-1)
    ex = Executors(ctx)
    yield ctx, ex
    ex.destroy()
    ctx.destroy()


def drain(ex, n, timeout_s=5.0):
    out = []
    for _ in range(n):
        r = ex.next_result(timeout_s)
        assert r is not None, "missing result"
        out.append(r)
    return out


def test_actions_wait_for_earliest_and_run_in_that_order(planning):
    ctx, ex = planning
    m = ctx.model_define_resnet(18, 64, 64)
    t0 = ex.now_ns()
    # submitted out of order; the executor must begin them by `earliest`
    for aid, delay in ((1, 60), (2, 20), (3, 40)):
        ex.submit(aid, CW_ACTION_UNLOAD, m, t0 + delay * MS, t0 + (delay + 500) * MS)
    res = drain(ex, 3)
    assert [r["id"] for r in res] == [2, 3, 1]
    for r, delay in zip(res, (20, 40, 60)):
        assert r["status"] == cw.CW_OK and r["type"] == CW_ACTION_UNLOAD
        assert t0 + delay * MS <= r["begin_ns"] <= t0 + (delay + 500) * MS    # inside its window, never early
        assert r["begin_ns"] - (t0 + delay * MS) < 15 * MS                    # and promptly (generous: shared test hosts)
        assert r["end_ns"] >= r["begin_ns"] and r["device_ns"] == 0
    assert ex.next_result(0.05) is None                                        # exactly one result each


def test_an_action_reached_after_latest_is_rejected_not_executed(planning):
    ctx, ex = planning
    m = ctx.model_define_resnet(18, 64, 64)
    t0 = ex.now_ns()
    ex.submit(7, CW_ACTION_UNLOAD, m, t0 - 20 * MS, t0 - 10 * MS)             # window already over
    ex.submit(8, CW_ACTION_UNLOAD, m, t0, t0 + 200 * MS)
    res = {r["id"]: r for r in drain(ex, 2)}
    assert res[7]["status"] == cw.CW_ERR_TOO_LATE and res[7]["end_ns"] == res[7]["begin_ns"]
    assert res[8]["status"] == cw.CW_OK
    # a blocked executor skips what it could not start in time and gets back on schedule (section 4.4):
    # the first action holds the UNLOAD executor until 80 ms, the second one's window closes at 40 ms
    t0 = ex.now_ns()
    ex.submit(10, CW_ACTION_UNLOAD, m, t0 + 80 * MS, t0 + 120 * MS)
    ex.submit(11, CW_ACTION_UNLOAD, m, t0 + 80 * MS, t0 + 80 * MS)           # a window of zero length behind it
    ex.submit(12, CW_ACTION_UNLOAD, m, t0 + 81 * MS, t0 + 200 * MS)
    res = {r["id"]: r for r in drain(ex, 3)}
    assert res[10]["status"] == cw.CW_OK and res[12]["status"] == cw.CW_OK
    assert res[11]["status"] == cw.CW_ERR_TOO_LATE                            # reached some microseconds after its latest


def test_device_actions_fail_cleanly_without_a_device_and_malformed_ones_are_refused(planning):
    ctx, ex = planning
    m = ctx.model_define_resnet(18, 64, 64)
    now = ex.now_ns()
    blob = np.zeros(ctx.model_weight_bytes(m), np.uint8)
    x = np.zeros((1, 3, 64, 64), np.float32)
    probs = np.zeros((1, 1000), np.float32)
    ex.submit(1, CW_ACTION_LOAD, m, now, now + 1000 * MS, host_in=blob)
    ex.submit(2, CW_ACTION_INFER, m, now, now + 1000 * MS, batch=1, host_in=x, host_probs=probs)
    res = {r["id"]: r for r in drain(ex, 2)}
    assert res[1]["status"] == cw.CW_ERR_INVALID and res[2]["status"] == cw.CW_ERR_INVALID   # planning-only context
    with pytest.raises(cw.CwError):
        ex.submit(3, 99, m, now, now + MS)                                    # unknown type
    with pytest.raises(cw.CwError):
        ex.submit(4, CW_ACTION_UNLOAD, m, now + MS, now)                      # latest before earliest
    with pytest.raises(cw.CwError):
        ex.submit(5, CW_ACTION_INFER, m, now, now + MS, batch=1, host_in=x)   # no output buffer
    assert ex.profile(CW_ACTION_UNLOAD, m)["n"] == 0


def test_profile_keeps_the_last_ten(planning):
    ctx, ex = planning
    m = ctx.model_define_resnet(18, 64, 64)
    now = ex.now_ns()
    for i in range(14):
        ex.submit(i, CW_ACTION_UNLOAD, m, now, now + 1000 * MS)
    res = drain(ex, 14)
    assert all(r["status"] == cw.CW_OK for r in res)
    p = ex.profile(CW_ACTION_UNLOAD, m)
    assert p["n"] == 10 and 0 <= p["mean_ns"] <= p["max_ns"] < 50 * MS


def test_destroy_with_pending_actions_returns():
    ctx = cw.Context(device=-1)
    ex = Executors(ctx)
    m = ctx.model_define_resnet(18, 64, 64)
    far = ex.now_ns() + 3600 * 1000 * MS
    for i in range(5):
        ex.submit(i, CW_ACTION_UNLOAD, m, far, far + MS)
    t = time.time()
    ex.destroy()
    assert time.time() - t < 2.0
    ctx.destroy()


@pytest.mark.gpu
def test_load_and_infer_actions_on_the_gpu():
    """LOAD, then INFERs with windows, through the executors: logits within tolerance of the CPU
    oracle (and bit for bit those of the direct calls, which run the same plan), EXEC begins inside
    its window, a late INFER is skipped and its slot comes back."""
    import torch
    from gpu_common import TOL, Case, rel_err_per_sample
    from oracle import network as N
    from oracle import topology as T
    from paper_2006_02464_amd.runner import Worker
    wk = Worker(workspace_bytes=64 << 20, io_bytes=32 << 20, weight_pool_bytes=64 << 20, load_staging_bytes=32 << 20)
    ctx = wk.ctx
    case = Case(T.resnet(18), 64, seed=0, dist="uniform")
    mid = ctx.model_define_resnet(18, 64, 64)
    x = case.images(0, 4)
    wk.load(mid, case.blob)
    direct = wk.infer(mid, x)                       # (probs, logits, ns) through the plain calls
    ref = case.oracle(x)                            # the CPU oracle on the same seeded tensors
    ctx.unload_weights(mid)
    ex = Executors(ctx)
    try:
        blob = torch.from_numpy(case.blob.copy()).pin_memory()
        hx = torch.from_numpy(x.copy()).pin_memory()
        now = ex.now_ns()
        ex.submit(100, CW_ACTION_LOAD, mid, now, now + 500 * MS, host_in=blob)
        r = ex.next_result(10.0)
        assert r["id"] == 100 and r["status"] == cw.CW_OK and r["device_ns"] > 0 and r["end_ns"] > r["begin_ns"]
        outs = {}
        now = ex.now_ns()
        for i in range(6):
            outs[i] = (torch.empty((4, 1000), dtype=torch.float32).pin_memory(), torch.empty((4, 1000), dtype=torch.float32).pin_memory())
            ex.submit(i, CW_ACTION_INFER, mid, now + (10 + 2 * i) * MS, now + (10 + 2 * i + 50) * MS, batch=4, host_in=hx,
                      host_probs=outs[i][0], host_logits=outs[i][1])
        late = (torch.empty((4, 1000), dtype=torch.float32).pin_memory(), None)
        ex.submit(50, CW_ACTION_INFER, mid, now - 5 * MS, now - 4 * MS, batch=4, host_in=hx, host_probs=late[0])
        res = {}
        for _ in range(7):
            r = ex.next_result(10.0)
            assert r is not None
            res[r["id"]] = r
        assert res[50]["status"] == cw.CW_ERR_TOO_LATE
        for i in range(6):
            r = res[i]
            assert r["status"] == cw.CW_OK
            assert now + (10 + 2 * i) * MS <= r["begin_ns"] <= now + (10 + 2 * i + 50) * MS
            assert 20_000 < r["device_ns"] < 5 * MS and r["end_ns"] - r["begin_ns"] >= r["device_ns"]
            assert rel_err_per_sample(outs[i][1].numpy(), ref["logits"]).max() <= TOL
            assert np.array_equal(N.argmax(outs[i][1].numpy()), N.argmax(ref["logits"]))
            assert np.abs(outs[i][0].numpy() - N.softmax(outs[i][1].numpy())).max() <= 1e-6
            assert np.array_equal(outs[i][1].numpy(), direct[1])      # same plan, same kernels: bit for bit
            assert np.array_equal(outs[i][0].numpy(), direct[0])
        p = ex.profile(CW_ACTION_INFER, mid, 4)
        assert p["n"] == 6 and p["max_ns"] >= p["mean_ns"] > 0
        now = ex.now_ns()
        ex.submit(200, CW_ACTION_UNLOAD, mid, now, now + 100 * MS)
        assert ex.next_result(5.0)["status"] == cw.CW_OK
        ex.submit(201, CW_ACTION_INFER, mid, now, now + 1000 * MS, batch=4, host_in=hx, host_probs=outs[0][0])
        assert ex.next_result(5.0)["status"] == cw.CW_ERR_NOT_LOADED
    finally:
        ex.destroy()
    # every IO slot came back (the rejected and the failed INFER released theirs)
    slots = [ctx.input(mid, 16, torch.zeros((16, 3, 64, 64)).pin_memory(), wk.stream) for _ in range(4)]
    for s in slots:
        ctx.release(s)
    wk.close()
