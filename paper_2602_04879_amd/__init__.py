"""DPPO divergence trust-region loss for MI355X (gfx950): hand-written HIP kernels behind a
C-ABI library, plus a thin ctypes binding.  Importing the package loads nothing; the HIP
library is opened on first use by `paper_2602_04879_amd.binding`."""

__all__ = ["binding", "autograd", "workloads", "build"]
