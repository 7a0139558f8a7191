"""Ring Reduce-Scatter / All-Gather / All-Reduce over simulated ranks on one MI355X.

The compute path is libhcl.so (hand-written HIP for gfx950) behind the C ABI in
include/hcl.h; `hcl` is its ctypes binding.  There is no CPU or PyTorch
fallback: calling into the binding without the built library raises.
"""
from . import hcl  # noqa: F401

__all__ = ["hcl"]
