"""Comparison helpers for the GPU parity tests: tolerances of the four result classes.

  rotated activations   max_j |gpu - oracle| <= 1e-5 * max_j |oracle| per token
  int4 codes            equal except +-1 flips where the oracle's scaled value sits within 5e-4 of a
                        rounding tie, on at most 1e-4 of the codes (at least one flip is tolerated on
                        small inputs)
  int32 accumulators    bit-exact
  bf16 outputs          |gpu - oracle| <= 1e-2 * |oracle| given identical codes and scales
"""
import numpy as np
import torch

import oracle


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
    assert np.all(dist < 5e-4), f"a flipped code is not at a rounding tie (distance {dist.max():.3e})"
    assert n <= max(1, int(frac * q_ref.size)), f"{n} flipped codes of {q_ref.size}"
    return n


def check_bf16(y_gpu: np.ndarray, y_ref: np.ndarray, tol: float = 1e-2):
    y_gpu = y_gpu.astype(np.float64)
    err = np.abs(y_gpu - y_ref)
    assert np.all(err <= tol * np.abs(y_ref)), f"bf16 output mismatch, worst rel {np.max(err / np.maximum(np.abs(y_ref), 1e-300)):.3e}"


def unpack_gpu(qx: torch.Tensor, signed: bool = True) -> np.ndarray:
    return oracle.unpack_int4(qx.cpu().numpy(), signed=signed)
