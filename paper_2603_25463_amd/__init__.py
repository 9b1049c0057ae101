"""MI355X-native CIAR quantify + verify hot path: HIP kernels behind a C ABI, with a thin binding.

``binding`` marshals torch tensors into the C ABI declared in ``include/ciar.h``;
``workloads`` generates the seeded synthetic inputs; ``build`` compiles ``libciar.so`` for gfx950.
"""
from .binding import (ENSEMBLE, VOTING, CiarError, Params, dense_intervals, finish_rows, last_error, lib, quantify,
                      quantify_multihead, quantify_verify, read_rows, stream_rows, verify, version, window_epilogue, workspace_bytes)

__all__ = ["ENSEMBLE", "VOTING", "CiarError", "Params", "dense_intervals", "finish_rows", "last_error", "lib", "quantify",
           "quantify_multihead", "quantify_verify", "read_rows", "stream_rows", "verify", "version", "window_epilogue", "workspace_bytes"]
