"""MI355X-native melded FP8-LoRA linear layer (hot path of FALQON, arXiv 2510.24061).

The compute lives in libfalqon.so (hand-written HIP for gfx950, C ABI in include/falqon.h).
This package is a thin ctypes binding with the same four names; PyTorch is used only to own
device memory and streams.
"""
from .binding import (  # noqa: F401
    E4M3, E5M2, BF16, F32, FalqonError, MeldedLinear, adamw_delta, da, db_bf16, fp8_gemm, grad_sqnorm, init_residual,
    lib, lib_path, melded_bwd, melded_fwd, proxy_update, proxy_update_static, row_score_bytes, quantize, status_string, svd_right_factor,
    svd_workspace_bytes, workspace_bytes,
)
