"""Pins for the oracle's MXFP4 quantizer and GEMM (no GPU): the OCP MX specification's element table,
hand-worked roundings and scales, error bounds of the format, and the block dot-product identity."""
import os

import numpy as np

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "mx_e2m1.txt")


def _fixture():
    table, ties = {}, []
    with open(GOLD) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            parts = line.split()
            if parts[0] == "tie":
                ties.append((float(parts[1]), float(parts[2])))
            else:
                table[int(parts[0], 2)] = float(parts[1])
    return table, ties


def test_e2m1_table_matches_the_specification():
    table, _ = _fixture()
    for code, value in table.items():
        assert oracle.e2m1_decode(np.array([code]))[0] == value
    # format arithmetic written out: (-1)^s 2^(E-1) (1 + M/2) for E > 0, (-1)^s 2^0 (M/2) for E = 0
    for code in range(16):
        s, E, M = code >> 3, (code >> 1) & 3, code & 1
        want = (M / 2.0) if E == 0 else 2.0 ** (E - 1) * (1 + M / 2.0)
        assert oracle.e2m1_decode(np.array([code]))[0] == (-want if s else want)


def test_e2m1_rounding_hand_values():
    _, ties = _fixture()
    for v, want in ties:
        got = oracle.e2m1_decode(oracle.e2m1_round(np.array([v])))[0]
        assert got == want, (v, got, want)
    # every representable value converts to itself
    vals = np.concatenate([oracle.E2M1_VALUES, -oracle.E2M1_VALUES[1:]])
    assert np.array_equal(oracle.e2m1_decode(oracle.e2m1_round(vals)), vals)
    # monotone and nearest: brute force over a fine grid against the value table
    grid = np.linspace(-7, 7, 28001)
    dec = oracle.e2m1_decode(oracle.e2m1_round(grid))
    allv = np.sort(np.concatenate([oracle.E2M1_VALUES, -oracle.E2M1_VALUES[1:]]))
    nearest_dist = np.min(np.abs(np.clip(grid, -6, 6)[:, None] - allv[None, :]), axis=1)
    assert np.allclose(np.abs(np.clip(grid, -6, 6) - dec), nearest_dist, atol=1e-12)
    assert np.all(np.diff(dec) >= 0)


def test_block_scale_hand_examples():
    def one(amax):
        x = np.zeros((1, 32))
        x[0, 5] = amax
        x[0, 6] = -amax / 3
        q, e = oracle.quantize_mxfp4(x)
        return int(e[0, 0]) - 127, oracle.dequantize_mxfp4(q, e)[0, 5]
    assert one(6.0) == (0, 6.0)           # floor(log2 6) = 2 -> X = 2^0, 6 is representable
    assert one(7.9) == (0, 6.0)           # still X = 1, 7.9 saturates to 6
    assert one(8.0) == (1, 8.0)           # floor(log2 8) = 3 -> X = 2, 8 / 2 = 4
    assert one(0.75) == (-3, 0.75)        # floor(log2 .75) = -1 -> X = 1/8, .75 * 8 = 6
    assert one(1.0) == (-2, 1.0)
    q, e = oracle.quantize_mxfp4(np.zeros((2, 64)))
    assert np.all(e == 0) and np.all(q == 0)
    # scales are per block of 32 along the row, blocks independent
    x = np.zeros((1, 64))
    x[0, 0] = 1.0
    x[0, 40] = 1024.0
    q, e = oracle.quantize_mxfp4(x)
    assert list(e[0]) == [127 - 2, 127 + 8]


def test_quantization_error_bound():
    rng = np.random.default_rng(0)
    x = rng.standard_t(3, size=(64, 256))
    q, e = oracle.quantize_mxfp4(x)
    assert q.dtype == np.uint8 and q.max() <= 15 and e.shape == (64, 8)
    dq = oracle.dequantize_mxfp4(q, e)
    X = np.repeat(np.ldexp(1.0, e.astype(np.int64) - 127), 32, axis=1)
    r = np.abs(x) / X
    # spacing of E2M1 is 0.5 below 2, 1 below 4, 2 below 6; beyond 6 (up to < 8) the value saturates
    bound = np.where(r < 2, 0.25, np.where(r < 4, 0.5, np.where(r <= 6, 1.0, 2.0))) * X
    assert np.all(np.abs(x - dq) <= bound * (1 + 1e-12))
    assert np.all(r < 8)
    # the block maximum lands in the top binade of the element format
    amax_r = np.max(r.reshape(64, 8, 32), axis=2)
    assert np.all((amax_r >= 4) & (amax_r < 8))


def test_pack_roundtrip_and_nibble_order():
    assert list(oracle.pack_fp4(np.array([1, 15, 8, 2], dtype=np.uint8))) == [0xF1, 0x28]
    rng = np.random.default_rng(1)
    c = rng.integers(0, 16, size=(5, 64), dtype=np.uint8)
    assert np.array_equal(oracle.unpack_fp4(oracle.pack_fp4(c)), c)


def test_gemm_is_the_block_scaled_dot_product():
    rng = np.random.default_rng(2)
    qx = rng.integers(0, 16, size=(3, 64), dtype=np.uint8)
    qw = rng.integers(0, 16, size=(4, 64), dtype=np.uint8)
    ex = rng.integers(120, 130, size=(3, 2), dtype=np.uint8)
    ew = rng.integers(120, 130, size=(4, 2), dtype=np.uint8)
    y = oracle.gemm_mxfp4(qx, ex, qw, ew)
    for t in range(3):
        for n in range(4):
            s = 0.0
            for blk in range(2):
                inner = 0.0
                for i in range(32):
                    inner += oracle.e2m1_decode(qx[t, 32 * blk + i:32 * blk + i + 1])[0] * \
                        oracle.e2m1_decode(qw[n, 32 * blk + i:32 * blk + i + 1])[0]
                s += 2.0 ** (int(ex[t, blk]) - 127) * 2.0 ** (int(ew[n, blk]) - 127) * inner
            assert y[t, n] == oracle.round_to_bf16(np.array([s]))[0]


def test_mxfp4_layer_tracks_the_unquantized_layer():
    rng = np.random.default_rng(3)
    N, M, Np = 64, 96, 32            # 96 = 12 * 8: a Paley base of order 12
    X = rng.standard_normal((40, N))
    W = rng.standard_normal((N, Np)) / 8
    qx, ex = oracle.quantize_mxfp4(oracle.rotate_structured(X, M))
    qw, ew = oracle.quantize_mxfp4(oracle.expand_weight(W, M).T)
    y = oracle.gemm_mxfp4(qx, ex, qw, ew)
    ref = X @ W
    assert np.linalg.norm(y - ref) / np.linalg.norm(ref) < 0.2
