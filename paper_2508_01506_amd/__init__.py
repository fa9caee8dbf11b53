"""fsvd: rank-aware streaming execution of one SVD-compressed transformer layer on MI355X.

`binding` wraps the C-ABI library (libfsvd.so, built by `build`); `workloads`
generates the seeded synthetic inputs.  There is no CPU or PyTorch fallback:
calling an entry point without the built library raises.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding", "build"]
