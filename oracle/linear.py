"""Integer GEMM, dequantising epilogue, the whole expanded layer, and the offline weight side.

Test infrastructure, fp64 / int64.  Section 3: at inference Q(X_hat) Q(W_hat) is computed,
with X_hat = X H_hat (online) and W_hat = H_hat^T W (offline), and X_hat W_hat = X W before
quantization.  Weights are stored as the transpose of the paper's W_hat: one row of M codes
per output channel, shape N' x M.
"""
from __future__ import annotations

import numpy as np

from .hadamard import expanded_hadamard, rotate_structured
from .quant import quantize_sym_int4, quantize_asym_int4, round_to_bf16


def int_gemm(qx: np.ndarray, qw: np.ndarray) -> np.ndarray:
    """acc[t, n] = sum_j qx[t, j] * qw[n, j], exact, int64.

    Evaluated as an fp64 matrix product of the integer codes: every partial sum is an
    integer of magnitude at most 15 * 8 * M < 2^53, so the fp64 result is exact.
    """
    a = np.asarray(qx).astype(np.float64)
    b = np.asarray(qw).astype(np.float64)
    return np.rint(a @ b.T).astype(np.int64)


def int_gemm_bruteforce(qx: np.ndarray, qw: np.ndarray) -> np.ndarray:
    """The same sum as three Python loops over Python integers (tiny inputs only)."""
    D, M = qx.shape
    Np = qw.shape[0]
    out = np.zeros((D, Np), dtype=np.int64)
    for t in range(D):
        for n in range(Np):
            s = 0
            for j in range(M):
                s += int(qx[t, j]) * int(qw[n, j])
            out[t, n] = s
    return out


def dequant_bf16(acc: np.ndarray, sx: np.ndarray, sw: np.ndarray) -> np.ndarray:
    """y[t, n] = bf16(acc[t, n] * sx[t] * sw[n]): the product in fp64, one rounding to bf16."""
    y = acc.astype(np.float64) * sx.astype(np.float64)[:, None] * sw.astype(np.float64)[None, :]
    return round_to_bf16(y)


def dequant_asym_bf16(acc: np.ndarray, sx: np.ndarray, zx: np.ndarray, qw: np.ndarray,
                      sw: np.ndarray) -> np.ndarray:
    """Asymmetric activations: x_j ~ sx (q_j - z), so y = sx sw (acc - z * sum_j qw[n, j])."""
    wsum = np.asarray(qw).astype(np.int64).sum(axis=1)
    corr = acc.astype(np.int64) - zx.astype(np.int64)[:, None] * wsum[None, :]
    return dequant_bf16(corr, sx, sw)


def expanded_linear(X: np.ndarray, M: int, qw: np.ndarray, sw: np.ndarray, asymmetric: bool = False):
    """The whole hot path for activations X (D x N): rotate, quantize, integer GEMM, dequantise.

    Returns a dict with every intermediate: xhat (fp64 D x M), qx, sx (and zx), acc (int64), y (fp64
    holding bf16 values).
    """
    xhat = rotate_structured(X, M)
    if asymmetric:
        qx, sx, zx = quantize_asym_int4(xhat)
        acc = int_gemm(qx, qw)
        y = dequant_asym_bf16(acc, sx, zx, qw, sw)
        return dict(xhat=xhat, qx=qx, sx=sx, zx=zx, acc=acc, y=y)
    qx, sx = quantize_sym_int4(xhat)
    acc = int_gemm(qx, qw)
    y = dequant_bf16(acc, sx, sw)
    return dict(xhat=xhat, qx=qx, sx=sx, acc=acc, y=y)


def expand_weight(W: np.ndarray, M: int) -> np.ndarray:
    """Offline weight expansion W_hat = H_hat^T W (Section 3).  W: N x N' -> M x N', fp64."""
    W = np.asarray(W, dtype=np.float64)
    return expanded_hadamard(W.shape[0], M).T @ W


def quantize_weight_rtn(What: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    """Per-output-channel symmetric int4 round-to-nearest of W_hat (M x N').

    Returns codes int8 [N', M] (transposed storage) in [-8, 7] and fp32 scales [N'];
    scale = absmax / 7 per output channel, same rounding rules as the activation quantizer.
    """
    q, s = quantize_sym_int4(np.asarray(What, dtype=np.float64).T)
    return q, s
