"""Seeded synthetic workloads for the expanded W4A4 linear layer.

This module only draws random inputs; it holds none of the method's arithmetic
(no Hadamard, no quantizer, no GEMM, no nibble packing).  Both the CPU oracle's
tests and the HIP path's tests / benchmark take their inputs from here so that
the two sides see identical data without sharing any code of the method.

The shapes are Llama-3 1B / 8B linear-layer shapes with the expanded inner
dimension d_e = b * 2^k; the activation statistics (Gaussian or heavy-tailed
Student-t rows with a small set of outlier channels scaled up) stand in for
the LLM activations that the paper quantizes (Sections 3 and 4), which need
model weights and a text corpus that are not available here.

Draw order for every workload (NumPy PCG64, `default_rng(seed)`):
activations -> outlier channel set -> weight codes -> weight scales.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    T: int                 # tokens (paper: D samples)
    d: int                 # input features (paper: N)
    d_e: int               # expanded features (paper: M)
    N: int                 # output channels (paper: N')
    in_dtype: str          # "f32" or "bf16"
    act_dist: str          # "normal" or "student_t3"
    outlier_frac: float    # fraction of channels scaled up (ignored if outlier_channels set)
    outlier_gain: float
    scale_lo: float
    scale_hi: float
    seed: int = 0
    outlier_channels: tuple = ()   # explicit channel list (Tiny)


SPECS = {
    "C1": WorkloadSpec("C1", 16, 64, 80, 64, "f32", "normal", 0.0, 50.0, 0.001, 0.01,
                       outlier_channels=(3, 17)),
    "C2": WorkloadSpec("C2", 2048, 2048, 2176, 3072, "bf16", "normal", 0.01, 50.0, 0.001, 0.01),
    "C3": WorkloadSpec("C3", 2048, 8192, 8704, 2048, "bf16", "student_t3", 0.005, 100.0, 0.001, 0.01),
    "C4": WorkloadSpec("C4", 8, 8192, 8448, 2048, "bf16", "normal", 0.01, 50.0, 0.001, 0.01),
    "C5": WorkloadSpec("C5", 4096, 14336, 15360, 4096, "bf16", "student_t3", 0.005, 100.0, 0.0005, 0.005),
}


@dataclass
class Workload:
    spec: WorkloadSpec
    x: np.ndarray            # [T, d] float32; for in_dtype == "bf16" every value is bf16-representable
    qw: np.ndarray           # [N, d_e] int8 codes in [-8, 7] (unpacked)
    sw: np.ndarray           # [N] float32 per-output-channel scales
    outliers: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))


def _to_bf16_grid(x32: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 value (ties to even); result stays float32."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def custom_spec(T: int, d: int, d_e: int, N: int, in_dtype: str = "bf16", act_dist: str = "normal",
                outlier_frac: float = 0.01, outlier_gain: float = 50.0,
                scale_lo: float = 0.001, scale_hi: float = 0.01, seed: int = 0,
                name: str = "custom") -> WorkloadSpec:
    return WorkloadSpec(name, T, d, d_e, N, in_dtype, act_dist, outlier_frac, outlier_gain,
                        scale_lo, scale_hi, seed)


def make_workload(spec, weights: bool = True) -> Workload:
    """Generate the tensors of one workload.  `spec` is a key of SPECS or a WorkloadSpec."""
    if isinstance(spec, str):
        spec = SPECS[spec]
    rng = np.random.default_rng(spec.seed)
    T, d = spec.T, spec.d
    if spec.act_dist == "normal":
        x = rng.standard_normal((T, d), dtype=np.float32)
    elif spec.act_dist == "student_t3":
        x = rng.standard_t(3.0, size=(T, d)).astype(np.float32)
    else:
        raise ValueError(spec.act_dist)
    if spec.outlier_channels:
        ch = np.asarray(spec.outlier_channels, dtype=np.int64)
    else:
        n_out = int(round(spec.outlier_frac * d))
        ch = np.sort(rng.choice(d, size=n_out, replace=False)) if n_out > 0 else np.zeros(0, np.int64)
    if ch.size:
        x[:, ch] *= np.float32(spec.outlier_gain)
    if spec.in_dtype == "bf16":
        x = _to_bf16_grid(x)
    elif spec.in_dtype != "f32":
        raise ValueError(spec.in_dtype)
    if weights:
        qw = rng.integers(-8, 8, size=(spec.N, spec.d_e), dtype=np.int8)
        sw = rng.uniform(spec.scale_lo, spec.scale_hi, size=spec.N).astype(np.float32)
    else:
        qw = np.zeros((0, spec.d_e), np.int8)
        sw = np.zeros(0, np.float32)
    return Workload(spec, x, qw, sw, ch)


def algorithmic_bytes_rotate_quant(spec: WorkloadSpec) -> int:
    """Bytes the rotate+quantize stage must move: read x, write packed codes and one scale per token."""
    in_size = 4 if spec.in_dtype == "f32" else 2
    return spec.T * (spec.d * in_size + spec.d_e // 2 + 4)


def gemm_ops(spec: WorkloadSpec) -> int:
    """Integer multiply-adds (counted as 2 ops) of the expanded GEMM."""
    return 2 * spec.T * spec.d_e * spec.N


def algorithmic_bytes_gemm(spec: WorkloadSpec) -> int:
    return spec.T * spec.d_e // 2 + spec.N * spec.d_e // 2 + 2 * spec.T * spec.N + 4 * (spec.T + spec.N)
