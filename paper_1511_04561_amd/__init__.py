"""dq8: the 8-bit approximation codec of arXiv 1511.04561 as hand-written HIP kernels for gfx950.

``paper_1511_04561_amd.dq8`` is the Python binding of the C-ABI library (argument
marshalling only); ``paper_1511_04561_amd.workloads`` generates the seeded synthetic
inputs.  Importing the package loads nothing; the shared library is loaded on the
first call and a missing library is an error, never a fallback.
"""
__all__ = ["dq8", "workloads"]
