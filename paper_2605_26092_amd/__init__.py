"""MI355X-native dual power-of-two linear-layer kernels (GoQuant hot path).

Thin Python binding over the C ABI of include/goq.h.  Every step of the path runs in the HIP
library (libgoq.so, built in-tree by paper_2605_26092_amd/build.py); this package only marshals
pointers.  torch is used for device memory and streams, nothing else.
"""
from .binding import (A3, A4, A6, A16, A8, F16, F32, GEMV_AUTO, GEMV_ROWS, GEMV_STREAM, GoqError, gemm, gemm_batch, gemm_folded, gemv,
                      gemv_batch, gemv_batch_ws, gemv_plan, gemv_select, gemv_stream, gemv_stream_table, gemv_workspace_bytes,
                      gemv_workspace_init, last_error, lib, mfma_probe, mfma_rate_probe, pack, packed_bytes, quantize, read_probe,
                      ref_coefficients, ref_workspace_bytes, unpack, version)

__all__ = ["A3", "A4", "A6", "A16", "A8", "F16", "F32", "GEMV_AUTO", "GEMV_ROWS", "GEMV_STREAM", "GoqError", "gemm", "gemm_batch", "gemm_folded", "gemv",
           "gemv_batch", "gemv_batch_ws", "gemv_plan", "gemv_select", "gemv_stream", "gemv_stream_table", "gemv_workspace_bytes", "gemv_workspace_init", "last_error", "lib", "mfma_probe", "mfma_rate_probe", "pack", "packed_bytes", "quantize", "read_probe", "ref_coefficients", "ref_workspace_bytes", "unpack", "version"]
