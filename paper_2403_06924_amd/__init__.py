"""srq: sparse-residual-compensated INT8 GEMM for MI355X (gfx950).

The compute lives in a C-ABI HIP library (``csrc/``, declared in
``include/srq.h``); :mod:`paper_2403_06924_amd.binding` marshals arguments to it.
Importing this package does not load the library; the binding does, and fails
loudly if it has not been built.
"""
__all__ = ["workloads"]
