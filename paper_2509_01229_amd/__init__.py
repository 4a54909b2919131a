"""MI355X-native LiquidQuant W4A8 GEMM: Python binding over the C-ABI HIP library.

Importing the package loads nothing; `paper_2509_01229_amd.api` loads the built shared
library on first use and raises if it is missing (there is no CPU fallback).
`paper_2509_01229_amd.workloads` holds the seeded synthetic input generators.
"""
__all__ = ["api", "workloads"]
