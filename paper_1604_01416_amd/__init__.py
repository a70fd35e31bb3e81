"""MI355X-native local GEMM and forward convolution (the per-GPU kernels of dMath).

``from paper_1604_01416_amd import dmath`` gives the thin ctypes binding over the
C-ABI library declared in ``include/dmath.h``.  ``workloads`` holds the seeded
synthetic input generators.  Importing the package itself loads nothing native.
"""
__all__ = ["dmath", "workloads"]
