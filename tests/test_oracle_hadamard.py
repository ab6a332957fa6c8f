"""Pins for the oracle's Hadamard construction and rotation (no GPU).

Each test checks the oracle against something fixed outside of it: a library routine,
a hand-worked fixture, an identity stated in Section 3 / Remarks 1-2 of the paper, or
brute force from the definition.
"""
import os

import numpy as np
import pytest
import scipy.linalg

import oracle
from workloads import make_workload

GOLD = os.path.join(os.path.dirname(__file__), "golden")
ORDERS = (80, 2176, 8704, 8448, 15360)
BASES = (12, 20, 60, 68, 72, 132, 140, 152, 312, 344)


def _signs(line):
    return [1 if ch == "+" else -1 for ch in line if ch in "+-"]


# ---------------------------------------------------------------- Sylvester block
@pytest.mark.parametrize("k", range(0, 9))
def test_sylvester_equals_scipy(k):
    # Textbook special case: natural-order Sylvester matrix is what scipy builds.
    S = oracle.sylvester(k)
    assert np.array_equal(S, scipy.linalg.hadamard(1 << k, dtype=np.int64))
    assert np.array_equal(S @ S.T, (1 << k) * np.eye(1 << k, dtype=np.int64))


# ---------------------------------------------------------------- Legendre symbol / Paley block
def test_legendre_matches_hand_worked_residues():
    with open(os.path.join(GOLD, "quadratic_residues.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            q, rest = line.split(":")
            q = int(q)
            residues = {int(v) for v in rest.split()}
            # brute force, independent of Euler's criterion used by the oracle
            assert residues == {(i * i) % q for i in range(1, q)}
            for a in range(-q, 2 * q):
                want = 0 if a % q == 0 else (1 if a % q in residues else -1)
                assert oracle.legendre_symbol(a, q) == want


def test_paley_order4_matches_hand_fixture():
    with open(os.path.join(GOLD, "paley_p4.txt")) as f:
        rows = [_signs(l) for l in f if not l.startswith("#") and l.strip()]
    assert np.array_equal(oracle.paley_block(4), np.array(rows))


def test_paley_order20_row1_matches_hand_fixture():
    with open(os.path.join(GOLD, "paley_p20_row1.txt")) as f:
        row = _signs(f.read())
    assert list(oracle.paley_block(20)[1]) == row


@pytest.mark.parametrize("b", BASES)
def test_paley_block_is_hadamard(b):
    P = oracle.paley_block(b)
    assert P.shape == (b, b)
    assert set(np.unique(P)) == {-1, 1}
    assert np.array_equal(P @ P.T, b * np.eye(b, dtype=np.int64))
    assert np.array_equal(P.T @ P, b * np.eye(b, dtype=np.int64))
    # structure of I + S with S skew: first row +1, first column (+1, -1, ...), unit diagonal
    assert np.all(P[0] == 1)
    assert P[0, 0] == 1 and np.all(P[1:, 0] == -1)
    assert np.all(np.diag(P) == 1)
    S = P - np.eye(b, dtype=np.int64)
    assert np.array_equal(S, -S.T)
    Q = S[1:, 1:]
    if b != 344:
        # over a prime field the Jacobsthal part is circulant: Q[i][j] depends on (i - j) mod q only
        assert np.array_equal(Q, np.roll(np.roll(Q, 1, axis=0), 1, axis=1))
    else:
        # over GF(7^3) it depends on the field difference x_i - x_j only
        from oracle.hadamard import gf343_sub
        q = b - 1
        diff = np.array([[gf343_sub(i, j) for j in range(q)] for i in range(q)])
        assert np.array_equal(Q, Q[:, 0][diff])


def test_gf343_is_a_field_of_order_343():
    from oracle.hadamard import gf343_mul, gf343_sub, gf343_quadratic_character
    # the modulus t^3 + t + 1 has no root in GF(7): a cubic without roots is irreducible
    assert all((t ** 3 + t + 1) % 7 != 0 for t in range(7))
    t, t2 = 7, 49                                  # element numbers of t and t^2
    assert gf343_mul(t, t) == t2
    assert gf343_mul(t, t2) == 6 + 6 * 7           # t^3 = -t - 1 = 6 + 6 t
    assert gf343_mul(t2, t2) == 6 * 7 + 6 * 49     # t^4 = -t^2 - t
    assert gf343_sub(0, 1) == 6 and gf343_sub(3, 3) == 0 and gf343_sub(7, 8) == 6
    # no zero divisors, and x -> x y is a bijection for y != 0 (checked for a few y)
    for y in (1, 2, 7, 50, 342):
        assert sorted(gf343_mul(x, y) for x in range(343)) == list(range(343))
    # the multiplicative group has order 342: x^342 = 1; a generator exists (t + 1 or another small element)
    def power(x, n):
        r = 1
        while n:
            if n & 1:
                r = gf343_mul(r, x)
            x = gf343_mul(x, x)
            n >>= 1
        return r
    assert all(power(x, 342) == 1 for x in range(1, 343))
    chi = gf343_quadratic_character()
    assert chi[0] == 0 and int((chi == 1).sum()) == 171 and int((chi == -1).sum()) == 171
    # Euler's criterion: chi(x) = x^((q-1)/2), and -1 is a non-square since q = 3 (mod 4)
    assert all((power(x, 171) == 1) == (chi[x] == 1) for x in range(1, 343))
    assert chi[gf343_sub(0, 1)] == -1


def test_paley_rejects_bad_orders():
    for b in (16, 22, 10, 36):   # q = 15 composite, 21 composite, 9 composite, 35 composite
        with pytest.raises(ValueError):
            oracle.paley_block(b)
    with pytest.raises(ValueError):
        oracle.paley_block(14)   # q = 13 is prime but 1 mod 4


# ---------------------------------------------------------------- factorisation
def test_factor_order_gives_the_workload_factorisations():
    assert oracle.factor_order(80) == (20, 2)
    assert oracle.factor_order(2176) == (68, 5)
    assert oracle.factor_order(8704) == (68, 7)
    assert oracle.factor_order(8448) == (132, 6)
    assert oracle.factor_order(15360) == (60, 8)
    assert oracle.factor_order(4096) == (1, 12)
    # layer sizes of Tables 1-2 that a Paley-I base covers
    assert oracle.factor_order(8960) == (140, 6)
    assert oracle.factor_order(9728) == (152, 6)
    assert oracle.factor_order(10240) == (20, 9)
    assert oracle.factor_order(12288) == (12, 10)
    assert oracle.factor_order(18432) == (72, 8)
    assert oracle.factor_order(19968) == (312, 6)
    assert oracle.factor_order(22016) == (344, 6)
    for bad in (7, 100, 11264):
        with pytest.raises(ValueError):
            oracle.factor_order(bad)


# ---------------------------------------------------------------- full matrix H
@pytest.mark.parametrize("M", (80, 2176, 64, 96))
def test_hadamard_full_orthogonality_small(M):
    H = oracle.hadamard_matrix(M)
    assert set(np.unique(H)) == {-1, 1}
    assert np.array_equal(H @ H.T, M * np.eye(M, dtype=np.int64))


@pytest.mark.parametrize("M", (8448, 8704, 15360))
def test_hadamard_sampled_rows_orthogonal_large(M):
    # H H^T = M I checked for 192 sampled rows against every row (exact in fp32: |sum| <= M < 2^24).
    H = oracle.hadamard_matrix(M).astype(np.int8)
    rng = np.random.default_rng(M)
    rows = np.sort(rng.choice(M, size=192, replace=False))
    G = H[rows].astype(np.float32) @ H.astype(np.float32).T
    want = np.zeros_like(G)
    want[np.arange(rows.size), rows] = M
    assert np.array_equal(G, want)


def test_kron_index_convention():
    # H[a 2^k + c, a' 2^k + c'] = P[a, a'] S[c, c'] spelled out entry by entry on the Tiny order.
    H = oracle.hadamard_matrix(80)
    P = oracle.paley_block(20)
    S = oracle.sylvester(2)
    for i in range(80):
        for j in range(80):
            assert H[i, j] == P[i // 4, j // 4] * S[i % 4, j % 4]


@pytest.mark.parametrize("N,M", ((64, 80), (2048, 2176), (50, 80)))
def test_expanded_hadamard_properties(N, M):
    Hh = oracle.expanded_hadamard(N, M)
    assert Hh.shape == (N, M)
    gamma = 1.0 / np.sqrt(M)
    # entries are +-gamma (Section 3)
    assert np.allclose(np.abs(Hh), gamma, rtol=0, atol=1e-17)
    # left inverse by transposition: H_hat H_hat^T = I_N (Section 3)
    assert np.allclose(Hh @ Hh.T, np.eye(N), rtol=0, atol=1e-12)
    # every column has norm sqrt(N / M) (Remark 2)
    assert np.allclose(np.linalg.norm(Hh, axis=0), np.sqrt(N / M), rtol=1e-13)
    # it is the first N rows of the M x M matrix, not the first N columns
    assert np.array_equal(np.sign(Hh).astype(np.int64), oracle.hadamard_matrix(M)[:N, :])


# ---------------------------------------------------------------- rotation
def _rotate_bruteforce(X, M):
    """x_hat_j = gamma * sum_{i < N} x_i H[i][j], loops straight from Section 3."""
    H = oracle.hadamard_matrix(M)
    D, N = X.shape
    out = np.zeros((D, M))
    for t in range(D):
        for j in range(M):
            s = 0.0
            for i in range(N):
                s += X[t, i] * H[i, j]
            out[t, j] = s / np.sqrt(M)
    return out


def test_rotate_bruteforce_tiny():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((3, 64))
    ref = _rotate_bruteforce(X, 80)
    assert np.allclose(oracle.rotate_explicit(X, 80), ref, rtol=0, atol=1e-13)
    assert np.allclose(oracle.rotate_structured(X, 80), ref, rtol=0, atol=1e-13)


def test_rotate_one_hot_gives_row_of_H_not_column():
    # e_i H_hat = gamma * (row i of H).  P_b is not symmetric, so using H^T would fail here.
    M, N = 80, 64
    H = oracle.hadamard_matrix(M)
    assert not np.array_equal(H, H.T)
    for i in (1, 5, 63):
        e = np.zeros((1, N))
        e[0, i] = 1.0
        for fn in (oracle.rotate_explicit, oracle.rotate_structured):
            got = fn(e, M)[0] * np.sqrt(M)
            assert np.allclose(got, H[i, :], atol=1e-12)
            assert not np.allclose(got, H[:, i], atol=1e-12)


@pytest.mark.parametrize("N,M,D", ((64, 80, 16), (2048, 2176, 4), (8192, 8448, 2), (300, 2176, 3),
                                   (14336, 15360, 1)))
def test_structured_equals_explicit(N, M, D):
    # includes a d that is not a multiple of 2^k (300): padding then ends inside a base row
    rng = np.random.default_rng(N + M)
    X = rng.standard_normal((D, N)) * (1 + 50 * (rng.random(N) < 0.01))
    a = oracle.rotate_explicit(X, M)
    b = oracle.rotate_structured(X, M)
    assert np.max(np.abs(a - b)) <= 1e-12 * np.max(np.abs(a))


def test_ratio_one_reduces_to_walsh_hadamard():
    # Expansion ratio 1.0 with a power-of-two width is the plain normalised Walsh-Hadamard transform.
    rng = np.random.default_rng(7)
    X = rng.standard_normal((5, 256))
    want = X @ scipy.linalg.hadamard(256) / 16.0
    assert np.allclose(oracle.rotate_structured(X, 256), want, atol=1e-12)
    assert np.allclose(oracle.rotate_explicit(X, 256), want, atol=1e-12)


def test_energy_preserved_and_rank_preserved():
    # ||X H_hat||_F = ||X||_F (Remark 2), rank(X_hat) = rank(X), nullity grows by M - N (Remark 1).
    wl = make_workload("C1", weights=False)
    X = wl.x.astype(np.float64)
    Xh = oracle.rotate_structured(X, 80)
    assert np.allclose(np.linalg.norm(Xh, axis=1), np.linalg.norm(X, axis=1), rtol=1e-13)
    assert np.isclose(np.linalg.norm(Xh), np.linalg.norm(X), rtol=1e-13)
    rng = np.random.default_rng(3)
    Xlow = rng.standard_normal((40, 7)) @ rng.standard_normal((7, 64))   # rank 7
    assert np.linalg.matrix_rank(Xlow) == 7
    assert np.linalg.matrix_rank(oracle.rotate_structured(Xlow, 80)) == 7


@pytest.mark.parametrize("N,M", ((64, 80), (2048, 2176)))
def test_computational_invariance(N, M):
    # X_hat W_hat = X H_hat H_hat^T W = X W (Section 3), unquantized.
    rng = np.random.default_rng(11)
    X = rng.standard_normal((6, N)) * (1 + 30 * (rng.random(N) < 0.02))
    W = rng.standard_normal((N, 24))
    What = oracle.expand_weight(W, M)
    assert What.shape == (M, 24)
    Y = oracle.rotate_structured(X, M) @ What
    ref = X @ W
    assert np.max(np.abs(Y - ref)) <= 1e-11 * np.max(np.abs(ref))
