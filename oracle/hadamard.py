"""Hadamard matrices of order M = b * 2^k and the expanded rotation X_hat = X H_hat.

Test infrastructure (see the package docstring).  Everything is fp64 / exact integers.

Section 3 of the paper defines H_hat as the first N rows of an M x M Hadamard matrix H
with entries +-gamma, gamma = 1/sqrt(M), so that H_hat H_hat^T = I_N, and the online
expansion as X_hat = X H_hat (X is D x N, X_hat is D x M).  The paper does not say how to
build H for an order that is not a power of two; the construction fixed for this build is
H = P_b (x) S_{2^k}: a Paley type-I block of order b (Kronecker) the Sylvester block of
order 2^k, with matrix index i = a * 2^k + c.
"""
from __future__ import annotations

import numpy as np

# Base orders b = q + 1 with q a prime (or, for 344, the prime power 7^3), q = 3 (mod 4), keyed by the
# odd part of b.  b = 1 is the pure power-of-two case (expansion ratio 1.0 in Section 4).
SUPPORTED_BASE = (1, 12, 20, 60, 68, 72, 132, 140, 152, 312, 344)


def sylvester(k: int) -> np.ndarray:
    """S_{2^k}: S_1 = [1], S_{2m} = [[S_m, S_m], [S_m, -S_m]] (natural order).  int64 entries +-1."""
    S = np.ones((1, 1), dtype=np.int64)
    for _ in range(k):
        S = np.block([[S, S], [S, -S]])
    return S


def legendre_symbol(a: int, q: int) -> int:
    """chi(a) over GF(q), q an odd prime: 0 if q | a, +1 if a is a non-zero square mod q, else -1."""
    a %= q
    if a == 0:
        return 0
    return 1 if pow(a, (q - 1) // 2, q) == 1 else -1


# GF(7^3) = GF(7)[t] / (t^3 + t + 1); the cubic has no root in GF(7), hence is irreducible.  Element number
# e = c0 + 7 c1 + 49 c2 stands for c0 + c1 t + c2 t^2.
GF343_P, GF343_MODULUS = 7, (1, 1, 0, 1)          # coefficients of 1 + t + 0 t^2 + t^3


def gf343_digits(e: int) -> tuple[int, int, int]:
    return e % 7, (e // 7) % 7, e // 49


def gf343_sub(e: int, f: int) -> int:
    """Number of the field element e - f (coefficient-wise, mod 7)."""
    a, b = gf343_digits(e), gf343_digits(f)
    c = [(x - y) % 7 for x, y in zip(a, b)]
    return c[0] + 7 * c[1] + 49 * c[2]


def gf343_mul(e: int, f: int) -> int:
    """Number of the field element e f: polynomial product, then t^3 = -t - 1 twice (degrees 4 and 3)."""
    a, b = gf343_digits(e), gf343_digits(f)
    prod = [0] * 5
    for i in range(3):
        for j in range(3):
            prod[i + j] += a[i] * b[j]
    for deg in (4, 3):                 # t^deg = t^(deg-3) t^3 = -(t^(deg-2) + t^(deg-3))
        c = prod[deg]
        prod[deg] = 0
        prod[deg - 2] -= c
        prod[deg - 3] -= c
    c = [v % 7 for v in prod[:3]]
    return c[0] + 7 * c[1] + 49 * c[2]


def gf343_quadratic_character() -> np.ndarray:
    """chi over GF(343) by element number: 0 at zero, +1 at the non-zero squares, -1 elsewhere."""
    chi = -np.ones(343, dtype=np.int64)
    chi[0] = 0
    for e in range(1, 343):
        chi[gf343_mul(e, e)] = 1
    return chi


def paley_block(b: int) -> np.ndarray:
    """Paley type-I Hadamard matrix of order b = q + 1, q = 3 (mod 4) a prime or 7^3.

    Jacobsthal matrix Q[i][j] = chi(x_i - x_j) over GF(q), the elements numbered 0 .. q-1 (a prime field:
    the residues; GF(343): see above); skew matrix S = [[0, 1^T], [-1, Q]]; P_b = I + S.
    b = 1 returns [[1]].  int64 entries +-1.
    """
    if b == 1:
        return np.ones((1, 1), dtype=np.int64)
    q = b - 1
    Q = np.empty((q, q), dtype=np.int64)
    if q == 343:
        chi = gf343_quadratic_character()
        for i in range(q):
            for j in range(q):
                Q[i, j] = chi[gf343_sub(i, j)]
    else:
        if q % 4 != 3 or any(q % p == 0 for p in range(2, int(q ** 0.5) + 1)):
            raise ValueError(f"order {b}: q = {q} is not a prime congruent to 3 mod 4")
        for i in range(q):
            for j in range(q):
                Q[i, j] = legendre_symbol(i - j, q)
    S = np.zeros((b, b), dtype=np.int64)
    S[0, 1:] = 1
    S[1:, 0] = -1
    S[1:, 1:] = Q
    return np.eye(b, dtype=np.int64) + S


def factor_order(M: int) -> tuple[int, int]:
    """Split M = b * 2^k with b the smallest supported base order dividing M with a power-of-two cofactor."""
    for b in SUPPORTED_BASE:
        if M % b == 0:
            c = M // b
            if c >= 1 and (c & (c - 1)) == 0:
                return b, c.bit_length() - 1
    raise ValueError(f"no supported factorisation b * 2^k for order {M}")


def hadamard_matrix(M: int) -> np.ndarray:
    """The +-1 Hadamard matrix H = P_b (x) S_{2^k} of order M (un-normalised, int64)."""
    b, k = factor_order(M)
    return np.kron(paley_block(b), sylvester(k))


def expanded_hadamard(N: int, M: int) -> np.ndarray:
    """H_hat = gamma * (first N rows of H), gamma = 1/sqrt(M); shape N x M, fp64 (Section 3)."""
    if not 0 < N <= M:
        raise ValueError("need 0 < N <= M")
    return hadamard_matrix(M)[:N, :].astype(np.float64) / np.sqrt(float(M))


def rotate_explicit(X: np.ndarray, M: int) -> np.ndarray:
    """X_hat = X H_hat with the explicit N x M matrix (Section 3).  X: D x N -> D x M, fp64."""
    X = np.asarray(X, dtype=np.float64)
    return X @ expanded_hadamard(X.shape[1], M)


def rotate_structured(X: np.ndarray, M: int) -> np.ndarray:
    """Same result as rotate_explicit through the Kronecker structure.

    With X~ = [X | 0] reshaped per token to b x 2^k (row a, column c, i = a 2^k + c),
    X_hat = gamma * P_b^T X~ S_{2^k}, because H[a 2^k + c, a' 2^k + c'] = P[a, a'] S[c, c'].
    """
    X = np.asarray(X, dtype=np.float64)
    D, N = X.shape
    b, k = factor_order(M)
    n = 1 << k
    Xp = np.zeros((D, M), dtype=np.float64)
    Xp[:, :N] = X
    Xt = Xp.reshape(D, b, n)
    P = paley_block(b).astype(np.float64)
    S = sylvester(k).astype(np.float64)
    Z = np.einsum("ap,tac->tpc", P, Xt)      # Z[t, a', c] = sum_a P[a, a'] X~[t, a, c]
    U = Z @ S                                # U[t, a', c'] = sum_c Z[t, a', c] S[c, c']
    return U.reshape(D, M) / np.sqrt(float(M))
