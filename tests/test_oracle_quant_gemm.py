"""Pins for the oracle's quantizers, packing, integer GEMM and bf16 epilogue (no GPU)."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from workloads import make_workload

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- symmetric quantizer
def test_tie_rounding_fixture():
    with open(os.path.join(GOLD, "tie_rounding.txt")) as f:
        lines = [l for l in f if not l.startswith("#")]
    x = np.array([float(v) for v in lines[0].split(":")[1].split()])[None, :]
    want = np.array([int(v) for v in lines[1].split(":")[1].split()])
    q, s = oracle.quantize_sym_int4(x)
    assert s.dtype == np.float32 and s[0] == np.float32(1.0)
    assert q.dtype == np.int8 and list(q[0]) == list(want)


def test_one_hot_closed_form():
    # e_i -> x_hat = gamma * H[i, :]: every entry has magnitude gamma, so codes = 7 sign(H[i, :]), s = gamma / 7.
    M, N = 80, 64
    H = oracle.hadamard_matrix(M)
    for i in (0, 1, 37):
        e = np.zeros((1, N))
        e[0, i] = 1.0
        q, s = oracle.quantize_sym_int4(oracle.rotate_structured(e, M))
        assert np.array_equal(q[0], 7 * H[i, :])
        assert s[0] == np.float32(1.0 / np.sqrt(M) / 7.0)


def test_zero_token_and_constant_magnitude():
    x = np.zeros((2, 8))
    x[1] = [3, -3, 3, 3, -3, -3, 3, -3]
    q, s = oracle.quantize_sym_int4(x)
    assert s[0] == 1.0 and np.all(q[0] == 0)
    assert s[1] == np.float32(3.0 / 7.0) and np.array_equal(q[1], 7 * np.sign(x[1]))


def test_quantizer_invariants_on_workload():
    wl = make_workload("C1", weights=False)
    xh = oracle.rotate_structured(wl.x, 80)
    q, s = oracle.quantize_sym_int4(xh)
    assert q.min() >= -7 and q.max() <= 7            # the clamp to [-8, 7] never fires with absmax / 7
    assert np.all(np.max(np.abs(q), axis=1) == 7)    # the absmax element maps to +-7
    err = np.abs(xh - s.astype(np.float64)[:, None] * q)
    assert np.all(err <= 0.5 * s.astype(np.float64)[:, None] * (1 + 1e-6))
    # scale is absmax/7 to fp32 precision
    assert np.allclose(s, np.max(np.abs(xh), axis=1) / 7.0, rtol=2 ** -23)


# ---------------------------------------------------------------- asymmetric quantizer (Section 4)
def test_asym_hand_example():
    # range [-3, 12] -> s = 1, z = 3; codes = rint(x) + 3
    x = np.array([[-3.0, 12.0, 0.0, 2.5, 3.5, -0.5, 7.49]])
    q, s, z = oracle.quantize_asym_int4(x)
    assert s[0] == 1.0 and z[0] == 3
    assert list(q[0]) == [0, 15, 3, 5, 7, 3, 10]


def test_asym_invariants():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((32, 80)) + 0.7
    x[3] = 0.0
    x[4] = np.abs(x[4])                      # all positive: range is widened to include 0
    q, s, z = oracle.quantize_asym_int4(x)
    assert q.min() >= 0 and q.max() <= 15 and z.min() >= 0 and z.max() <= 15
    assert s[3] == 1.0 and np.all(q[3] == z[3])
    assert z[4] == 0
    recon = s.astype(np.float64)[:, None] * (q.astype(np.float64) - z[:, None])
    # zero-point rounding moves the grid by at most half a step, rounding by another half
    assert np.all(np.abs(recon - x) <= s.astype(np.float64)[:, None] * (1.0 + 1e-6))


# ---------------------------------------------------------------- packing
def test_pack_hand_bytes():
    assert list(oracle.pack_int4(np.array([-8, 7, 1, -1, 0, 3], dtype=np.int8))) == [0x78, 0xF1, 0x30]
    assert list(oracle.unpack_int4(np.array([0x78, 0xF1, 0x30], dtype=np.uint8))) == [-8, 7, 1, -1, 0, 3]
    assert list(oracle.unpack_int4(np.array([0x78, 0xF1], dtype=np.uint8), signed=False)) == [8, 7, 1, 15]


def test_pack_roundtrip():
    rng = np.random.default_rng(2)
    q = rng.integers(-8, 8, size=(7, 80), dtype=np.int8)
    p = oracle.pack_int4(q)
    assert p.shape == (7, 40) and p.dtype == np.uint8
    assert np.array_equal(oracle.unpack_int4(p), q)
    u = rng.integers(0, 16, size=(7, 80), dtype=np.uint8)
    assert np.array_equal(oracle.unpack_int4(oracle.pack_int4(u), signed=False), u)


# ---------------------------------------------------------------- integer GEMM
def test_int_gemm_bruteforce_c1():
    wl = make_workload("C1")
    q, _ = oracle.quantize_sym_int4(oracle.rotate_structured(wl.x, 80))
    acc = oracle.int_gemm(q, wl.qw)
    assert acc.dtype == np.int64 and acc.shape == (16, 64)
    assert np.array_equal(acc, oracle.int_gemm_bruteforce(q, wl.qw))
    # orientation: weights are [N', M], contraction over M
    assert np.array_equal(acc, q.astype(np.int64) @ wl.qw.astype(np.int64).T)


def test_int_gemm_exact_at_extreme_codes():
    # worst-case magnitude 8 * 8 * M summed coherently stays exact
    M = 15360
    qx = np.full((2, M), -8, dtype=np.int8)
    qw = np.full((3, M), -8, dtype=np.int8)
    qw[1] = 7
    acc = oracle.int_gemm(qx, qw)
    assert np.array_equal(acc, np.array([[64 * M, -56 * M, 64 * M]] * 2))


def test_one_hot_gemm_closed_form():
    wl = make_workload("C1")
    H = oracle.hadamard_matrix(80)
    e = np.zeros((1, 64))
    e[0, 9] = 1.0
    out = oracle.expanded_linear(e, 80, wl.qw, wl.sw)
    want = 7 * (H[9, :][None, :] * wl.qw.astype(np.int64)).sum(axis=1)
    assert np.array_equal(out["acc"][0], want)


# ---------------------------------------------------------------- bf16 rounding / epilogue
def test_round_to_bf16_hand_values():
    v = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -30, -2.5 - 2.0 ** -7,
                  0.0, 3.0e38, 3.4e38, 2.0 ** -133, 2.0 ** -134, 1.5 * 2.0 ** -133])
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -2.5,
                     0.0, 2.9908e38, np.inf, 2.0 ** -133, 0.0, 2.0 ** -132])
    got = oracle.round_to_bf16(v)
    assert got[7] == np.inf
    mask = np.arange(v.size) != 6
    assert np.array_equal(got[mask], want[mask])
    assert abs(got[6] - 3.0e38) <= 2.0 ** 119      # within half a bf16 step of the input


def test_round_to_bf16_matches_torch_on_fp32_inputs():
    # For inputs that are exactly fp32, torch's fp32 -> bf16 conversion is the same single RNE rounding.
    rng = np.random.default_rng(9)
    v32 = np.concatenate([rng.standard_normal(200000).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 200000).astype(np.float32),
                          np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1e-40, -1e-39, 6e-41], dtype=np.float32)])
    want = torch.from_numpy(v32).to(torch.bfloat16).to(torch.float64).numpy()
    got = oracle.round_to_bf16(v32.astype(np.float64))
    assert np.array_equal(got, want)


def test_dequant_hand_example():
    acc = np.array([[100, -3], [0, 7]], dtype=np.int64)
    sx = np.array([0.5, 0.25], dtype=np.float32)
    sw = np.array([0.125, 2.0], dtype=np.float32)
    y = oracle.dequant_bf16(acc, sx, sw)
    assert np.array_equal(y, np.array([[6.25, -3.0], [0.0, 3.5]]))
    # 257 * 1 * 1 is not a bf16 number: ties-to-even gives 256
    assert oracle.dequant_bf16(np.array([[257]]), np.ones(1, np.float32), np.ones(1, np.float32))[0, 0] == 256.0
    assert oracle.dequant_bf16(np.array([[259]]), np.ones(1, np.float32), np.ones(1, np.float32))[0, 0] == 260.0


def test_dequant_asym_identity():
    # sx sw (acc - z sum_j qw) equals the product of the dequantised activations with the integer weights
    rng = np.random.default_rng(4)
    x = rng.standard_normal((5, 80)) + 0.3
    qw = rng.integers(-8, 8, size=(6, 80), dtype=np.int8)
    sw = rng.uniform(0.001, 0.01, 6).astype(np.float32)
    q, s, z = oracle.quantize_asym_int4(x)
    acc = oracle.int_gemm(q, qw)
    y = oracle.dequant_asym_bf16(acc, s, z, qw, sw)
    xdq = s.astype(np.float64)[:, None] * (q.astype(np.float64) - z[:, None])
    ref = oracle.round_to_bf16((xdq @ qw.astype(np.float64).T) * sw.astype(np.float64)[None, :])
    # both round once from fp64; products differ only in association
    assert np.max(np.abs(y - ref)) <= 2.0 ** -7 * np.max(np.abs(ref))
    assert np.mean(y == ref) > 0.99


# ---------------------------------------------------------------- whole layer
def test_expanded_linear_tracks_unquantized_layer():
    # Sanity of the end-to-end chain (the size of the quantization error itself is unpinned by the paper):
    # with weights obtained by expanding and RTN-quantizing a real W, the quantized layer approximates X W.
    rng = np.random.default_rng(21)
    N, M, Np = 64, 80, 32
    X = rng.standard_normal((64, N))
    W = rng.standard_normal((N, Np)) / 8.0
    qw, sw = oracle.quantize_weight_rtn(oracle.expand_weight(W, M))
    assert qw.shape == (Np, M) and sw.shape == (Np,) and qw.dtype == np.int8 and sw.dtype == np.float32
    y = oracle.expanded_linear(X, M, qw, sw)["y"]
    ref = X @ W
    rel = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    assert rel < 0.2
    ya = oracle.expanded_linear(X, M, qw, sw, asymmetric=True)["y"]
    assert np.linalg.norm(ya - ref) / np.linalg.norm(ref) < 0.2


def test_weight_quantizer_hand_example_is_per_output_channel_and_transposed():
    """Section 4: per-channel symmetric int4 weights.  W_hat is M x N' (rows = expanded input features, columns =
    output channels); the codes come back as one row per output channel.  Worked by hand: column 0 has absmax 3.5,
    so its scale is 0.5 and its codes are the entries doubled; column 1 has absmax 14, scale 2, codes entries / 2
    with 2.5 -> 2 and -0.5 -> 0 at the ties (round half to even)."""
    What = np.array([[3.5, 14.0], [-1.0, 5.0], [0.25, -1.0], [-3.5, 3.0]])
    q, s = oracle.quantize_weight_rtn(What)
    assert q.shape == (2, 4) and s.shape == (2,)
    assert np.array_equal(s, np.array([0.5, 2.0], dtype=np.float32))
    assert np.array_equal(q[0], [7, -2, 0, -7])          # 0.25 / 0.5 = 0.5 -> 0 (tie to even)
    assert np.array_equal(q[1], [7, 2, 0, 2])            # 2.5 -> 2, -0.5 -> -0, 1.5 -> 2
    # a scale per column, not per row: scaling one output channel changes only that channel's scale
    q2, s2 = oracle.quantize_weight_rtn(What * np.array([1.0, 4.0]))
    assert np.array_equal(q2, q) and np.array_equal(s2, np.array([0.5, 8.0], dtype=np.float32))
    # reconstruction error at most half a step per entry
    assert np.all(np.abs(q.T * s[None, :].astype(np.float64) - What) <= 0.5 * s[None, :] + 1e-12)


def test_c1_regression_fixture():
    with open(os.path.join(GOLD, "c1_oracle.json")) as f:
        g = json.load(f)
    wl = make_workload("C1")
    out = oracle.expanded_linear(wl.x, 80, wl.qw, wl.sw)
    assert [float(v) for v in out["sx"]] == g["sx"]
    assert int(out["qx"].astype(np.int64).sum()) == g["qx_sum"]
    assert int(np.abs(out["qx"].astype(np.int64)).sum()) == g["qx_abs_sum"]
    assert int(out["acc"].sum()) == g["acc_sum"]
    assert [int(v) for v in out["acc"][0, :8]] == g["acc_row0"]
    assert [float(v) for v in out["y"][0, :8]] == g["y_row0"]
