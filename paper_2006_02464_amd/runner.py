"""Small conveniences over the binding for harnesses: pinned host buffers and a
stream from PyTorch, one INFER = INPUT -> EXEC -> OUTPUT.  No arithmetic here."""
import numpy as np
import torch

from .binding import Context


def require_gpu():
    if not torch.cuda.is_available():
        raise RuntimeError("no GPU: the EXEC path has no CPU implementation")
    name = torch.cuda.get_device_properties(0).gcnArchName
    if not name.startswith("gfx950"):
        raise RuntimeError("kernels are built for gfx950 only, found %s" % name)


def pinned_like(arr):
    """Pinned host copy of a numpy array (returned as a torch tensor view)."""
    t = torch.empty(arr.shape, dtype=torch.from_numpy(arr[:0].copy()).dtype, pin_memory=True)
    t.numpy()[...] = arr
    return t


class Worker:
    """One context plus one stream; keeps pinned staging buffers alive."""

    def __init__(self, **ctx_kwargs):
        require_gpu()
        self.ctx = Context(**ctx_kwargs)
        self.stream = torch.cuda.Stream()
        self._keep = []

    def load(self, model_id, blob):
        pinned = pinned_like(np.ascontiguousarray(blob))
        self.ctx.load_weights(model_id, pinned, self.stream)
        self.stream.synchronize()

    def infer(self, model_id, x, classes=1000):
        """x: float32 [B][C][H][W] numpy.  Returns (probs, logits, exec_ns)."""
        b = x.shape[0]
        hx = pinned_like(np.ascontiguousarray(x, dtype=np.float32))
        probs = torch.empty((b, classes), dtype=torch.float32, pin_memory=True)
        logits = torch.empty((b, classes), dtype=torch.float32, pin_memory=True)
        slot = self.ctx.input(model_id, b, hx, self.stream)
        self.ctx.exec(model_id, b, slot, self.stream)
        ns = self.ctx.exec_duration_ns(slot)
        self.ctx.output(slot, probs, logits, self.stream)
        self.stream.synchronize()
        return probs.numpy().copy(), logits.numpy().copy(), ns

    def close(self):
        self.stream.synchronize()
        self.ctx.destroy()
