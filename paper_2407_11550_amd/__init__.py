"""MI355X-native Ada-KV per-layer cache compression: score, allocate, select, compact.

Decode side of the resulting flattened cache: cache_build, append, decode_attn, decode_step.
All calls run entirely in the HIP library (csrc/); this package only marshals
arguments.  Importing the package does not load the library; the first call does,
and raises if the library has not been built.
"""
from .binding import (PROBE_SINK_BYTES, STATIC_SCRATCH_BYTES, AdaKVError, KernelTrace, Layer, allocate, append, cache_build, cache_rows,  # noqa: F401
                      compact, compress, compress_static, decode_attn, decode_step, decode_workspace_bytes, describe, library_path,
                      load_library, probe_read, pyramid_budgets, score, select, workspace_bytes)
