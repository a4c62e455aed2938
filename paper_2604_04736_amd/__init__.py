"""MI355X-native mean-field Gaussian sample layer for sampling-parallel Bayesian learning.

The product is the HIP library ``libhot`` (``csrc/``, declared in ``include/hot.h``);
``binding`` marshals torch tensors into its C ABI, ``autograd`` wraps the sample layer as a
differentiable torch function, ``workloads`` makes seeded synthetic inputs.  Nothing is loaded at import time: the library is opened on first use and a
missing library is an error, never a fallback.
"""

__all__ = ["autograd", "binding", "workloads"]
