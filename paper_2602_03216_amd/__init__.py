"""Token Sparse Attention prefill hot path for MI355X (gfx950): hand-written HIP kernels behind
a C ABI (include/tsa.h), a ctypes binding of the same names (binding.py) and the seeded input
generator (inputs.py).  `binding` needs torch and the built libtsa.so and is imported on use."""
from . import inputs  # noqa: F401

__all__ = ["inputs"]
