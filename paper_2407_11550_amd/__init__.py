"""MI355X-native Ada-KV per-layer cache compression: score, allocate, select, compact.

The four calls run entirely in the HIP library (csrc/); this package only marshals
arguments.  Importing the package does not load the library; the first call does,
and raises if the library has not been built.
"""
from .binding import (AdaKVError, KernelTrace, Layer, allocate, compact, compress, library_path,  # noqa: F401
                      load_library, score, select, workspace_bytes)
