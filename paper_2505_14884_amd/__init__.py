"""MI355X-native Selective Head Attention decode path (router + top-k + selective decode attention).

The compute runs in hand-written HIP kernels behind a C-ABI library (``include/polar.h``);
``binding`` marshals torch device tensors into it and ``workloads`` generates seeded inputs.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads"]
