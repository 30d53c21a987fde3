"""MI355X-native bi-level / tri-level l1,q projection (arXiv 2405.02086).

The compute lives in csrc/ (hand-written gfx950 HIP kernels behind a C ABI,
declared in include/mlproj.h); `binding` marshals arguments for it.  Importing
the package loads nothing heavy: `workloads` (seeded inputs) is pure numpy and
`binding` opens the shared library on first use and fails loudly if it is absent.
"""
__all__ = ["binding", "workloads"]
