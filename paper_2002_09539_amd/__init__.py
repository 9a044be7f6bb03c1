"""Overlap Local-SGD hot path for one MI355X: HIP kernels behind a C boundary (libols.so).

`binding` mirrors include/ols.h one-to-one; `session` holds the device buffers and streams a run needs.
"""
from . import binding  # noqa: F401
