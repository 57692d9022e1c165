"""MI355X-native table-batched embedding-bag operator (forward + backward fused with row-wise AdaGrad).

`tbe` is the ctypes binding of the HIP library (csrc/, built into libtbe.so by `build`);
`workloads` generates the seeded synthetic inputs.  Nothing here computes on the CPU.
"""
from . import workloads  # noqa: F401
from . import tbe  # noqa: F401

__all__ = ["tbe", "workloads"]
