"""cw_exec_static, the EXEC entry point that allocates nothing: its intermediates live in an array
built into the library.  Called through the C ABI on two calls in a row, the second with a smaller
input, and compared with cw_exec (same plan, same kernels: bit for bit) and with the CPU oracle."""
import numpy as np
import pytest
import torch

import paper_2006_02464_amd as cw
from gpu_common import TOL, Case, rel_err_per_sample
from oracle import topology as T

pytestmark = pytest.mark.gpu


def _static_infer(wk, mid, x, classes=1000):
    xd = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
    logits = torch.full((x.shape[0], classes), float("nan"), device="cuda")
    probs = torch.full((x.shape[0], classes), float("nan"), device="cuda")
    torch.cuda.synchronize()                      # the buffers are ready before the EXEC stream uses them
    wk.ctx.exec_static(mid, x.shape[0], xd, logits, probs, wk.stream)
    wk.stream.synchronize()
    return probs.cpu().numpy(), logits.cpu().numpy()


def test_exec_static_matches_exec_on_two_calls_in_a_row():
    from paper_2006_02464_amd.runner import Worker
    wk = Worker(workspace_bytes=512 << 20, io_bytes=64 << 20, weight_pool_bytes=256 << 20, load_staging_bytes=64 << 20)
    try:
        ctx = wk.ctx
        assert ctx.exec_static_capacity() == 80 << 20
        # ResNet-50 at 224x224: batch 4, then batch 1 (split-K launches: partial sums and arrival
        # counters in the arena), then a ResNet-18 at 64x64 over the arena the others left behind
        r50 = Case(T.resnet(50), 224, seed=0, dist="normal")
        m50 = ctx.model_define_resnet(50, 224, 224)
        wk.load(m50, r50.blob)
        assert any(l["split_k"] > 1 for l in ctx.plan(m50, 1))
        x = r50.images(0, 4)
        ref = r50.oracle(x)["logits"]
        for first, count in ((0, 4), (1, 1), (0, 2)):
            xs = x[first:first + count]
            probs_e, logits_e, _ = wk.infer(m50, xs)
            probs_s, logits_s = _static_infer(wk, m50, xs)
            assert np.array_equal(logits_s, logits_e) and np.array_equal(probs_s, probs_e)
            assert rel_err_per_sample(logits_s, ref[first:first + count]).max() <= TOL
        # the largest plan of the metric's model (fused launches with their third layer): 68.6 MiB of the arena
        x16 = r50.images(0, 16)
        probs_e, logits_e, _ = wk.infer(m50, x16)
        probs_s, logits_s = _static_infer(wk, m50, x16)
        assert np.array_equal(logits_s, logits_e) and np.array_equal(probs_s, probs_e)
        assert np.array_equal(logits_s[:4], logits_e[:4]) and rel_err_per_sample(logits_s[:4], ref).max() <= TOL
        r18 = Case(T.resnet(18), 64, seed=0, dist="uniform")
        m18 = ctx.model_define_resnet(18, 64, 64)
        wk.load(m18, r18.blob)
        for count in (16, 2):
            xs = r18.images(0, count)
            probs_e, logits_e, _ = wk.infer(m18, xs)
            probs_s, logits_s = _static_infer(wk, m18, xs)
            assert np.array_equal(logits_s, logits_e) and np.array_equal(probs_s, probs_e)
            assert rel_err_per_sample(logits_s, r18.oracle(xs)["logits"]).max() <= TOL
        # errors: beyond the arena, not loaded, no plan, null buffer
        big = ctx.model_define(r50.ops, 3, 448, 448, batch_sizes=(16,))
        assert ctx.model_workspace_bytes(big, 16) > ctx.exec_static_capacity()
        wk.load(big, r50.blob)
        d = torch.zeros(16, device="cuda")
        with pytest.raises(cw.CwError) as e:
            ctx.exec_static(big, 16, d, d, d, wk.stream)
        assert e.value.status == cw.CW_ERR_NO_MEMORY and "static arena" in str(e.value)
        ctx.unload_weights(m18)
        with pytest.raises(cw.CwError) as e:
            ctx.exec_static(m18, 2, d, d, d, wk.stream)
        assert e.value.status == cw.CW_ERR_NOT_LOADED
        with pytest.raises(cw.CwError) as e:
            ctx.exec_static(m50, 3, d, d, d, wk.stream)
        assert e.value.status == cw.CW_ERR_BAD_BATCH
        with pytest.raises(cw.CwError) as e:
            ctx.exec_static(m50, 1, d, None, d, wk.stream)
        assert e.value.status == cw.CW_ERR_INVALID
        # and the arena still serves after the refused calls
        probs_s, logits_s = _static_infer(wk, m50, x[:1])
        assert rel_err_per_sample(logits_s, ref[:1]).max() <= TOL
    finally:
        wk.close()
