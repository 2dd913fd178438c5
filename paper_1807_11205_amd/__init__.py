"""libjz for MI355X: the single-GPU hot path of mixed-precision CNN training with LARS
(Jia et al. 2018, Section 4.1) as hand-written HIP kernels behind a C ABI.

Importing the package loads nothing; `paper_1807_11205_amd.api` opens the built library
and raises if it is missing.
"""
__all__ = ["api", "inputs", "shapes"]
