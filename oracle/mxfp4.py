"""OCP Microscaling MXFP4 quantizer and GEMM (the paper's second quantization setting, Section 4: OCP MXFP4
weights and activations, one E8M0 scale per group of 32 elements).  Test infrastructure, fp64.

Written from the public OCP Microscaling Formats (MX) specification v1.0:
 * element format FP4 E2M1: sign, 2 exponent bits (bias 1), 1 mantissa bit, no Inf/NaN; magnitudes by
   code 0..7: 0, 0.5, 1, 1.5, 2, 3, 4, 6;
 * shared scale E8M0 per block of 32 consecutive elements: X = 2^(byte - 127), byte 255 = NaN;
 * conversion of a block V: shared_exp = floor(log2(max_i |V_i|)) - emax_elem with emax_elem = 2, clamped
   to [-127, 127]; P_i = V_i / X rounded to the element format, here round-to-nearest-even, values beyond
   the largest magnitude saturating to +-6.  An all-zero block takes the smallest scale (byte 0).
 * dot product of two MX vectors: sum over blocks of X_a X_b sum_i P_a,i P_b,i.
"""
from __future__ import annotations

import numpy as np

from .quant import round_to_bf16

E2M1_VALUES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
BLOCK = 32


def e2m1_round(v: np.ndarray) -> np.ndarray:
    """Nearest E2M1 magnitude code (0..7) of |v| with ties to the even code, saturating; plus the sign bit (8)."""
    v = np.asarray(v, dtype=np.float64)
    a = np.abs(v)
    code = np.zeros(a.shape, dtype=np.uint8)
    # midpoints between consecutive magnitudes; a tie goes to the code with an even mantissa bit (even code)
    for c in range(7):
        mid = 0.5 * (E2M1_VALUES[c] + E2M1_VALUES[c + 1])
        up = (a > mid) | ((a == mid) & (c % 2 == 1))     # from an odd code the even neighbour is above
        code = np.where(up, c + 1, code).astype(np.uint8)
    code = np.where(np.signbit(v) & (a > 0), code | 8, code).astype(np.uint8)
    return code


def e2m1_decode(code: np.ndarray) -> np.ndarray:
    code = np.asarray(code).astype(np.int64)
    mag = E2M1_VALUES[code & 7]
    return np.where(code & 8, -mag, mag)


def quantize_mxfp4(X: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    """Rows of X (last dimension a multiple of 32) -> (codes uint8 [.., M] in 0..15, scale bytes uint8 [.., M/32])."""
    X = np.asarray(X, dtype=np.float64)
    D, M = X.shape
    if M % BLOCK:
        raise ValueError("the row length must be a multiple of 32")
    B = X.reshape(D, M // BLOCK, BLOCK)
    amax = np.max(np.abs(B), axis=2)
    # floor(log2) through frexp is exact for every positive double: amax = f 2^p, f in [0.5, 1) -> p - 1
    _, p = np.frexp(amax)
    e = np.where(amax > 0, p - 1, -127 + 2).astype(np.int64)
    shared = np.clip(e - 2, -127, 127)
    scale = np.ldexp(1.0, shared)
    codes = e2m1_round(B / scale[:, :, None]).reshape(D, M)
    return codes, (shared + 127).astype(np.uint8)


def dequantize_mxfp4(codes: np.ndarray, scale_bytes: np.ndarray) -> np.ndarray:
    codes = np.asarray(codes)
    D, M = codes.shape
    scale = np.ldexp(1.0, scale_bytes.astype(np.int64) - 127)
    return (e2m1_decode(codes).reshape(D, M // BLOCK, BLOCK) * scale[:, :, None]).reshape(D, M)


def pack_fp4(codes: np.ndarray) -> np.ndarray:
    """Two 4-bit codes per byte, even index in the low nibble."""
    codes = np.asarray(codes, dtype=np.uint8)
    return (codes[..., 0::2] | (codes[..., 1::2] << 4)).astype(np.uint8)


def unpack_fp4(p: np.ndarray) -> np.ndarray:
    p = np.asarray(p, dtype=np.uint8)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = p & 0xF
    out[..., 1::2] = p >> 4
    return out


def gemm_mxfp4(qx, ex, qw, ew, return_abs: bool = False):
    """y[t, n] = bf16(sum over blocks of X_x X_w sum_i P_x,i P_w,i), the sum in fp64, one rounding to bf16.

    With return_abs also the sum of the magnitudes of the terms (the scale of fp32 accumulation error)."""
    a = dequantize_mxfp4(qx, ex)
    b = dequantize_mxfp4(qw, ew)
    y = a @ b.T
    if return_abs:
        return round_to_bf16(y), np.abs(a) @ np.abs(b).T
    return round_to_bf16(y)
