"""Expanded W4A4 linear layer for MI355X: thin Python binding over the C-ABI library libpme.so.

Every step of the path runs in the library's HIP kernels; this package only marshals
arguments (torch tensors give device pointers and the current stream).  There is no CPU
or PyTorch fallback: if the library has not been built, importing the binding functions
raises.
"""
from .binding import (PmeError, lib, version, set_path, get_path, set_gemm_tile, factor_order, base_block, workspace_bytes,
                      hadamard_expand_quant, hadamard_expand_quant_asym, hadamard_expand_f32, expand_quantize_weights,
                      hadamard_expand_quant_mxfp4, mxfp4_gemm, expanded_linear_mxfp4,
                      w4a4_gemm, w4a4_gemm_asym, w4a4_gemm_i32, weight_rowsum, expanded_linear, expanded_linear_static, STATIC_SCRATCH_BYTES, expanded_linear_asym,
                      probe_copy, probe_read, probe_launch, probe_mfma, pack_int4, gemm_plan, PATH_AUTO, PATH_GENERIC, PATH_MFMA, EXPORTS)

__all__ = ["PmeError", "lib", "version", "set_path", "get_path", "set_gemm_tile", "factor_order", "base_block", "workspace_bytes",
           "hadamard_expand_quant", "hadamard_expand_quant_asym", "hadamard_expand_f32", "expand_quantize_weights", "hadamard_expand_quant_mxfp4", "mxfp4_gemm",
           "expanded_linear_mxfp4", "w4a4_gemm",
           "w4a4_gemm_asym", "w4a4_gemm_i32", "weight_rowsum", "expanded_linear", "expanded_linear_static", "STATIC_SCRATCH_BYTES", "expanded_linear_asym", "probe_copy", "probe_read", "probe_launch", "probe_mfma",
           "pack_int4", "gemm_plan", "PATH_AUTO", "PATH_GENERIC", "PATH_MFMA", "EXPORTS"]
