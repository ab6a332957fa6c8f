"""Comparison helpers for the GPU parity tests: tolerances of the four result classes.

  rotated activations   max_j |gpu - oracle| <= 1e-5 * max_j |oracle| per token
  int4 codes            equal except +-1 flips where the oracle's scaled value sits within 5e-5 of a
                        rounding tie, on at most 1e-4 of the codes (at least one flip is tolerated on
                        small inputs)
  int32 accumulators    bit-exact
  bf16 outputs          |gpu - oracle| <= 1e-2 * |oracle| given identical codes and scales
"""
import numpy as np
import torch

import oracle

# A code may differ from the oracle's only where the oracle's scaled value is this close (in code steps) to a
# half-integer: fp32 butterflies over k + log2(b) levels leave an error of a few 1e-7 of the token's absmax,
# i.e. a few 1e-6 code steps; the window leaves a factor of ten over that.
TIE_WINDOW = 5e-5


def to_device(x32: np.ndarray, in_dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x32))
    if in_dtype == "bf16":
        tb = t.to(torch.bfloat16)
        assert torch.equal(tb.to(torch.float32), t), "generator output must be bf16-representable"
        t = tb
    return t.cuda()


def check_xhat(gpu: np.ndarray, ref: np.ndarray, tol: float = 1e-5):
    err = np.max(np.abs(gpu.astype(np.float64) - ref), axis=1)
    scale = np.max(np.abs(ref), axis=1)
    bad = err > tol * scale + 1e-300
    assert not bad.any(), f"rotation mismatch on {bad.sum()} rows, worst rel {np.max(err / np.maximum(scale, 1e-300)):.3e}"
    return float(np.max(err / np.maximum(scale, 1e-300)))


def check_scales(gpu: np.ndarray, ref: np.ndarray, tol: float = 1e-5):
    rel = np.abs(gpu.astype(np.float64) - ref.astype(np.float64)) / np.abs(ref.astype(np.float64))
    assert np.all(rel <= tol), f"scale mismatch, worst rel {rel.max():.3e}"


def check_codes(q_gpu: np.ndarray, q_ref: np.ndarray, xhat_ref: np.ndarray, s_ref: np.ndarray, frac: float = 1e-4):
    diff = q_gpu.astype(np.int16) - q_ref.astype(np.int16)
    flips = diff != 0
    n = int(flips.sum())
    if n == 0:
        return 0
    assert np.all(np.abs(diff[flips]) == 1), "a code differs by more than one step"
    scaled = xhat_ref / s_ref.astype(np.float64)[:, None]
    dist = np.abs(np.abs(scaled[flips] - np.floor(scaled[flips])) - 0.5)
    assert np.all(dist < TIE_WINDOW), f"a flipped code is not at a rounding tie (distance {dist.max():.3e})"
    assert n <= max(1, int(frac * q_ref.size)), f"{n} flipped codes of {q_ref.size}"
    return n


def check_bf16(y_gpu: np.ndarray, y_ref: np.ndarray, tol: float = 1e-2):
    y_gpu = y_gpu.astype(np.float64)
    err = np.abs(y_gpu - y_ref)
    assert np.all(err <= tol * np.abs(y_ref)), f"bf16 output mismatch, worst rel {np.max(err / np.maximum(np.abs(y_ref), 1e-300)):.3e}"


def unpack_gpu(qx: torch.Tensor, signed: bool = True) -> np.ndarray:
    return oracle.unpack_int4(qx.cpu().numpy(), signed=signed)


def check_mx_quant(qx: torch.Tensor, ex: torch.Tensor, ref_x: np.ndarray):
    """Scale bytes equal except where the block maximum sits within 1e-5 of a power of two; on blocks with
    equal scales the codes are equal except neighbouring-value flips at rounding ties (<= 1e-4 of the codes)."""
    q_ref, e_ref = oracle.quantize_mxfp4(ref_x)
    q = oracle.unpack_fp4(qx.cpu().numpy())
    e = ex.cpu().numpy()
    D, M = ref_x.shape
    bad = e != e_ref
    if bad.any():
        amax = np.max(np.abs(ref_x.reshape(D, M // 32, 32)), axis=2)[bad]
        frac, _ = np.frexp(amax)
        assert np.all(np.minimum(np.abs(frac - 0.5), np.abs(frac - 1.0)) < 1e-5), "scale byte differs away from a power of two"
        assert np.all(np.abs(e.astype(int) - e_ref.astype(int))[bad] == 1)
        assert bad.sum() <= max(1, int(1e-5 * bad.size))
    same = np.repeat(~bad, 32, axis=1)
    flips = (q != q_ref) & same
    n = int(flips.sum())
    if n:
        X = np.repeat(np.ldexp(1.0, e_ref.astype(np.int64) - 127), 32, axis=1)
        scaled = np.abs(ref_x / X)[flips]
        mids = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
        dist = np.min(np.abs(scaled[:, None] - mids[None, :]), axis=1)
        assert np.all(dist < 5e-4), f"a flipped code is not at a rounding tie ({dist.max():.3e})"
        dec_gap = np.abs(oracle.e2m1_decode(q[flips]) - oracle.e2m1_decode(q_ref[flips]))
        assert np.all(dec_gap <= 2.0)
        assert n <= max(1, int(1e-4 * q.size)), f"{n} flipped codes of {q.size}"
    return n


def check_mx_gemm(y_gpu, qx, ex, qw, ew):
    """bf16 rounding (1e-2 relative) plus fp32 accumulation inside the matrix core, bounded by 2^-18 of the
    sum of the magnitudes of the terms (K <= 2^14 terms, error grows like sqrt(K) 2^-24 of that sum)."""
    y_ref, abs_sum = oracle.gemm_mxfp4(qx, ex, qw, ew, return_abs=True)
    err = np.abs(y_gpu.astype(np.float64) - y_ref)
    assert np.all(err <= 1e-2 * np.abs(y_ref) + 2.0 ** -18 * abs_sum), f"worst {np.max(err / (np.abs(y_ref) + 1e-30)):.3e}"
