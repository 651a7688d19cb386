"""MI355X-native FastKV token-importance selection (arXiv 2502.01068, Sec. 4.2 / App. B.1).

The compute lives in ``csrc/`` (HIP kernels for gfx950 behind the C ABI declared in
``include/fastkv_select.h``); ``binding`` marshals torch device tensors into it.  Importing
the package loads nothing; the shared library is opened on first use and a missing
library is an error, never a fallback.
"""
__all__ = ["binding", "workloads"]
