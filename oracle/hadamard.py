"""Hadamard matrices for the output transform (oracle side; test infrastructure).

Section 3.3: a Hadamard matrix has entries +-1 and H H^T = n I; the Walsh-Hadamard
family is H_{2^k} = H_2 (x) H_{2^{k-1}}; for n that is not a power of two, n = 2^p m with
m the order of a known Hadamard matrix.  The paper takes the m-order matrices from a
published table that is not available here; any Hadamard matrix satisfies the fold
identity of Section 4.2, so the orders 12 and 20 are built by the first Paley
construction (q = 11, 19 prime, q = 3 mod 4) straight from its definition.
"""
from __future__ import annotations

import numpy as np


def sylvester(m: int) -> np.ndarray:
    """H_{2^m} by the recursive block definition of Section 3.3 (int8 entries)."""
    H = np.ones((1, 1), dtype=np.int8)
    H2 = np.array([[1, 1], [1, -1]], dtype=np.int8)
    for _ in range(m):
        H = np.kron(H2, H)
    return H


def _legendre(a: int, q: int) -> int:
    a %= q
    if a == 0:
        return 0
    # Euler's criterion: a^((q-1)/2) mod q is 1 for residues, q-1 for non-residues
    return 1 if pow(a, (q - 1) // 2, q) == 1 else -1


def paley1(q: int) -> np.ndarray:
    """Hadamard matrix of order q+1 for a prime q = 3 (mod 4): H = I + S with S the
    skew matrix bordered by +1 (first row) / -1 (first column) around the Jacobsthal
    matrix Q[i, j] = chi(i - j)."""
    assert q % 4 == 3
    n = q + 1
    S = np.zeros((n, n), dtype=np.int64)
    S[0, 1:] = 1
    S[1:, 0] = -1
    for i in range(q):
        for j in range(q):
            S[i + 1, j + 1] = _legendre(i - j, q)
    H = np.eye(n, dtype=np.int64) + S
    return H.astype(np.int8)


def hadamard_factor(n: int):
    """(k, m) with n = k * 2^m, k in {1, 12, 20} (Section 3.3, n = 2^p m)."""
    odd, p = n, 0
    while odd % 2 == 0:
        odd //= 2
        p += 1
    if odd == 1:
        return 1, p
    if odd == 3 and p >= 2:
        return 12, p - 2
    if odd == 5 and p >= 2:
        return 20, p - 2
    raise ValueError(f"no Hadamard factorisation k*2^m with k in (1, 12, 20) for n={n}")


def hadamard_matrix(n: int) -> np.ndarray:
    """Dense H_n = H_k (x) H_{2^m}: entry [a*2^m + b, a'*2^m + b'] = H_k[a, a'] * H_{2^m}[b, b']."""
    k, m = hadamard_factor(n)
    Hk = {1: np.ones((1, 1), dtype=np.int8), 12: None, 20: None}[k]
    if k == 12:
        Hk = paley1(11)
    elif k == 20:
        Hk = paley1(19)
    return np.kron(Hk, sylvester(m)).astype(np.int8)
