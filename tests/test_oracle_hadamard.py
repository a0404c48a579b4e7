"""Pins for the oracle's Hadamard matrices (Section 3.3; fold identity of Section 4.2)."""
import os

import numpy as np
import pytest

from oracle import hadamard_factor, hadamard_matrix, paley1, sylvester

GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.mark.parametrize("name,m", [("sylvester_h2.txt", 1), ("sylvester_h4.txt", 2)])
def test_sylvester_matches_printed_seed(name, m):
    want = np.loadtxt(os.path.join(GOLD, name), dtype=np.int64)
    assert np.array_equal(sylvester(m).astype(np.int64), want)


@pytest.mark.parametrize("m", range(0, 9))
def test_sylvester_closed_form(m):
    n = 1 << m
    i = np.arange(n)
    pc = np.array([[bin(a & b).count("1") for b in i] for a in i])
    assert np.array_equal(sylvester(m).astype(np.int64), (-1) ** pc)


@pytest.mark.parametrize("q", [3, 7, 11, 19])
def test_paley_is_hadamard(q):
    H = paley1(q).astype(np.int64)
    n = q + 1
    assert set(np.unique(H)) == {-1, 1}
    assert np.array_equal(H @ H.T, n * np.eye(n, dtype=np.int64))
    assert np.array_equal(H.T @ H, n * np.eye(n, dtype=np.int64))


@pytest.mark.parametrize("n,km", [(1536, (12, 7)), (5120, (20, 8)), (8192, (1, 13)), (128, (1, 7)),
                                  (48, (12, 2)), (80, (20, 2)), (12, (12, 0)), (2048, (1, 11))])
def test_factorisation(n, km):
    assert hadamard_factor(n) == km
    assert km[0] * (1 << km[1]) == n


@pytest.mark.parametrize("n", [100, 6, 10, 7 * 64, 9 * 128])
def test_factorisation_rejects(n):
    with pytest.raises(ValueError):
        hadamard_factor(n)


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32, 64, 128, 256, 12, 20, 24, 40, 48, 96, 160, 1536, 5120,
                               8192])
def test_orthogonality_dense(n):
    H = hadamard_matrix(n)
    assert H.shape == (n, n)
    assert np.all(np.abs(H) == 1)
    Hf = H.astype(np.float32)  # sums are integers of magnitude <= n < 2^24: exact in fp32
    G = Hf @ Hf.T
    assert np.array_equal(G, np.float32(n) * np.eye(n, dtype=np.float32))


@pytest.mark.parametrize("n", [48, 1536, 5120])
def test_kronecker_index_rule(n):
    """H_n[a*2^m + b, a'*2^m + b'] = H_k[a, a'] * (-1)^popcount(b & b')."""
    k, m = hadamard_factor(n)
    H = hadamard_matrix(n)
    Hk = paley1(k - 1)
    rng = np.random.default_rng(0)
    for _ in range(2000):
        i, j = rng.integers(0, n, size=2)
        a, b, a2, b2 = i >> m, i & ((1 << m) - 1), j >> m, j & ((1 << m) - 1)
        assert H[i, j] == Hk[a, a2] * (-1) ** bin(b & b2).count("1")


@pytest.mark.parametrize("n", [12, 20, 48, 1536])
def test_not_symmetric_orientation(n):
    """The Paley factors are not symmetric, so H vs H^T matters: transforming the unit
    vector e_j must give column j of H (y^H = H y), not row j."""
    H = hadamard_matrix(n).astype(np.float64)
    assert not np.array_equal(H, H.T)
    j = 5
    e = np.zeros(n)
    e[j] = 1.0
    assert np.array_equal(H @ e, H[:, j])


@pytest.mark.parametrize("n", [48, 256, 1536])
def test_fold_identity(n):
    """W_out^T y = (1/n) (W_out^H)^T y^H with y^H = H y, W_out^H rows = H W_out rows."""
    rng = np.random.default_rng(1)
    W = rng.standard_normal((7, n))
    y = rng.standard_normal((5, n))
    y[0, 3] = 1e3
    H = hadamard_matrix(n).astype(np.float64)
    yH = y @ H.T
    WH = W @ H.T
    ref = y @ W.T
    got = (yH @ WH.T) / n
    assert np.max(np.abs(got - ref)) <= 1e-12 * np.max(np.abs(ref)) * n
    # the other orientation of the fold is wrong for the non-symmetric orders
    if n != 256:
        bad = (yH @ (W @ H).T) / n
        assert np.max(np.abs(bad - ref)) > 1e-3 * np.max(np.abs(ref))
