"""MI355X-native CIAR quantify + verify hot path: HIP kernels behind a C ABI, with a thin binding.

``binding`` marshals torch tensors into the C ABI declared in ``include/ciar.h``;
``workloads`` generates the seeded synthetic inputs; ``build`` compiles ``libciar.so`` for gfx950.
"""
from .binding import (DRO_LOSSES, DRO_TERMS, ENSEMBLE, VOTING, CiarError, Params, dense_intervals,
                      finish_rows, interdro_loss, interhead_logits, interhead_quantify, last_error, lib, quantify, quantify_multihead,
                      quantify_verify, quantify_verify_static, read_rows, stream_rows, verify, version, window_epilogue,
                      workspace_bytes)

__all__ = ["DRO_LOSSES", "DRO_TERMS", "ENSEMBLE", "VOTING", "CiarError", "Params", "dense_intervals",
           "finish_rows", "interdro_loss", "interhead_logits", "interhead_quantify", "last_error", "lib", "quantify", "quantify_multihead",
           "quantify_verify", "quantify_verify_static", "read_rows", "stream_rows", "verify", "version", "window_epilogue",
           "workspace_bytes"]
