"""DD-EF-SGD hot path on AMD MI355X: HIP kernels behind a C-ABI library, bound with ctypes.

`binding` loads libddef.so (built in tree by `build.build_library()`); `workloads` makes the
seeded synthetic inputs.  Importing the package loads nothing.
"""
__all__ = ["binding", "build", "workloads"]
