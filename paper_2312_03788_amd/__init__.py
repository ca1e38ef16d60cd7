"""SmoothQuant+ W4A16 linear layer for AMD MI355X: thin binding over libsqp.so.

Every operation runs in the HIP library; this package only marshals arguments
(torch tensors -> device pointers, current stream).  There is no CPU fallback:
if the library is missing or a call fails, an exception is raised.
"""
from .binding import (SqpError, alpha_search, interleave_gate_up, rmsnorm, scale_columns, w4a16_gemm_silu_mul, dequantize, lib, quantize_pack, quant_loss, smooth_apply_w,
                      smooth_apply_x, smooth_scales, transpose_nk, w4a16_gemm, set_workspace, workspace_bytes, w4a16_gemm_static)

__all__ = ["SqpError", "lib", "smooth_scales", "smooth_apply_x", "smooth_apply_w", "quantize_pack",
           "dequantize", "w4a16_gemm", "quant_loss", "alpha_search", "transpose_nk", "w4a16_gemm_silu_mul", "rmsnorm", "scale_columns", "interleave_gate_up", "set_workspace", "workspace_bytes", "w4a16_gemm_static"]
