"""librap for MI355X: thin Python binding over the C-ABI shared library.

The binding only marshals arguments (device pointers of torch tensors, the current HIP stream);
every step of the path runs in the HIP kernels of librap.so.  There is no fallback: if the
library has not been built, loading fails with an error that says how to build it.
"""
from __future__ import annotations

from .binding import Rap, RapError, RapPaging, RapShape, RapTuning, load, library_path  # noqa: F401

__all__ = ["Rap", "RapError", "RapPaging", "RapShape", "RapTuning", "load", "library_path"]
