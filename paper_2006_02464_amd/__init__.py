"""MI355X-native EXEC hot path of a Clockwork worker: thin ctypes binding over
libclockwork_exec.so (HIP kernels + C ABI).  There is no CPU fallback: without
the built library, or without a gfx950 GPU, device calls raise."""
from .binding import *  # noqa: F401,F403
