"""MI355X-native small-batch inference GeMM (hand-written HIP for gfx950 behind a C ABI).

`paper_2207_00032_amd.binding` is the thin ctypes face of libsbi_gemm.so;
`paper_2207_00032_amd.workloads` draws the seeded synthetic inputs.  Importing the package
loads nothing: the shared library is opened on the first call that needs it and a missing
library raises (there is no CPU fallback).
"""
__all__ = ["binding", "workloads"]
