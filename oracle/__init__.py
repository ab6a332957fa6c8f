"""CPU oracle for the expanded W4A4 linear layer (post-training model expansion, Section 3).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 NumPy statement of what
the hot path computes.  It shares no code with the HIP library or its Python binding and
imports neither.  Only tests, the smoke check and the benchmark's CPU-baseline leg may
import it; the product path never does.

Pinned parts (see tests/test_oracle_*.py): Sylvester block, Paley block, full and
expanded Hadamard matrix, rotation (explicit and structured), quantizer, integer GEMM,
bf16 epilogue, offline weight expansion, MXFP4 quantizer and GEMM.

Parity unpinned: the *value* of the quantized layer output relative to the unquantized
layer X W.  The paper gives no error bound for Q(X H) Q(H^T W) versus X W, so only
oracle-vs-HIP parity is judged for it.
"""
from .hadamard import (sylvester, legendre_symbol, paley_block, factor_order, hadamard_matrix,
                       expanded_hadamard, rotate_explicit, rotate_structured, SUPPORTED_BASE)
from .quant import (quantize_sym_int4, quantize_asym_int4, pack_int4, unpack_int4, round_to_bf16)
from .mxfp4 import (E2M1_VALUES, e2m1_round, e2m1_decode, quantize_mxfp4, dequantize_mxfp4, pack_fp4, unpack_fp4,
                    gemm_mxfp4)
from .linear import (int_gemm, int_gemm_bruteforce, dequant_bf16, dequant_asym_bf16, expanded_linear,
                     expand_weight, quantize_weight_rtn)
