"""Quantizers and number formats of the expanded W4A4 layer.  Test infrastructure, fp64.

Section 4 ("Quantization Details") uses per-channel symmetric int4 weights and per-token
int4 activations.  The hot path of this build quantizes activations per token
*symmetrically*; the paper's per-token asymmetric variant is provided as well.
The paper fixes neither the divisor of the symmetric range, the rounding mode nor the
precision of the stored scale.  Readings taken here: scale = absmax / 7 stored as fp32,
round half to even, clamp to [-8, 7], an all-zero token gets scale 1 and codes 0.
"""
from __future__ import annotations

import numpy as np


def quantize_sym_int4(Xhat: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    """Per-token (row) symmetric int4: returns (codes int8 [D, M] in [-8, 7], scale fp32 [D]).

    m = max_j |x_j|; s = fp32(m / 7) (1 if m == 0); q_j = clip(rint(x_j / s), -8, 7), the
    division done in fp64 by the fp32-rounded scale.
    """
    Xhat = np.asarray(Xhat, dtype=np.float64)
    m = np.max(np.abs(Xhat), axis=1)
    s = (m / 7.0).astype(np.float32)
    s = np.where(m == 0.0, np.float32(1.0), s).astype(np.float32)
    q = np.rint(Xhat / s.astype(np.float64)[:, None])
    q = np.clip(q, -8, 7).astype(np.int8)
    return q, s


def quantize_asym_int4(Xhat: np.ndarray) -> tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Per-token asymmetric uint4 (Section 4): returns (codes uint8 in [0, 15], scale fp32, zero-point int32).

    lo = min(min_j x_j, 0), hi = max(max_j x_j, 0) (the range always contains 0, as usual for an
    affine quantizer; the paper does not say); s = fp32((hi - lo) / 15) (1 if hi == lo);
    z = clip(rint(-lo / s), 0, 15); q_j = clip(rint(x_j / s) + z, 0, 15).  x_j ~ s (q_j - z).
    """
    Xhat = np.asarray(Xhat, dtype=np.float64)
    lo = np.minimum(Xhat.min(axis=1), 0.0)
    hi = np.maximum(Xhat.max(axis=1), 0.0)
    s = ((hi - lo) / 15.0).astype(np.float32)
    s = np.where(hi == lo, np.float32(1.0), s).astype(np.float32)
    s64 = s.astype(np.float64)
    z = np.clip(np.rint(-lo / s64), 0, 15).astype(np.int32)
    q = np.clip(np.rint(Xhat / s64[:, None]) + z[:, None], 0, 15).astype(np.uint8)
    return q, s, z


def pack_int4(q: np.ndarray) -> np.ndarray:
    """Two 4-bit codes per byte along the last axis: even index in the low nibble, odd in the high.

    Signed codes are stored as 4-bit two's complement, unsigned codes as they are.
    """
    q = np.asarray(q)
    if q.shape[-1] % 2:
        raise ValueError("last dimension must be even")
    u = (q.astype(np.int16) & 0xF).astype(np.uint8)
    return (u[..., 0::2] | (u[..., 1::2] << 4)).astype(np.uint8)


def unpack_int4(p: np.ndarray, signed: bool = True) -> np.ndarray:
    """Inverse of pack_int4."""
    p = np.asarray(p, dtype=np.uint8)
    lo = (p & 0xF).astype(np.int16)
    hi = (p >> 4).astype(np.int16)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.int16)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    if signed:
        out = np.where(out >= 8, out - 16, out)
        return out.astype(np.int8)
    return out.astype(np.uint8)


def round_to_bf16(v: np.ndarray) -> np.ndarray:
    """Round fp64 values once to the nearest bfloat16 (8 significand bits, ties to even).

    Returned as fp64 holding exactly the bf16 value.  Written from the format's definition:
    |v| = f * 2^e with f in [0.5, 1); the spacing of bf16 numbers there is 2^(e-8), but never
    below 2^-133 (subnormals); values that round beyond the largest finite bf16 become inf.
    """
    v = np.asarray(v, dtype=np.float64)
    f, e = np.frexp(v)
    e = np.maximum(e - 8, -133)
    r = np.ldexp(np.rint(np.ldexp(v, -e)), e)
    max_bf16 = (2.0 - 2.0 ** -7) * 2.0 ** 127
    r = np.where(np.abs(r) > max_bf16, np.copysign(np.inf, r), r)
    return np.where(np.isfinite(v), r, v)
