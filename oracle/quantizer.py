"""Symmetric uniform int8 quantizer and integer GEMM (oracle side; test infrastructure).

Section 3.2, Eq. 2: X_q = clamp(round(X / s), -2^(N-1), 2^(N-1)-1), s = max|X| / (2^(N-1)-1),
N = 8, s static.  Section 4.2 ("SSM inputs"): the scan input x uses the p-th percentile of
|x| in place of the maximum.  Sections 4.2 / 4.3 write the fused operators as a multiply by
1/s; the oracle follows that form: one fp32 multiply by a stored reciprocal (or a stored
product of scales), round to nearest with ties to even, clamp.
"""
from __future__ import annotations

import math

import numpy as np

QMIN, QMAX = -128, 127


def rne(v: np.ndarray) -> np.ndarray:
    """Round to nearest integer, ties to even."""
    return np.rint(v)


def quantize(v, inv_s) -> np.ndarray:
    """Eq. 2 in its fused form: clamp(rne(fp32(v) * fp32(1/s)), -128, 127) -> int8."""
    t = np.asarray(v, dtype=np.float32) * np.float32(inv_s)
    return np.clip(rne(t), QMIN, QMAX).astype(np.int8)


def requant_acc(acc, m) -> np.ndarray:
    """int32 accumulator -> int8: clamp(rne(fp32(acc) * m), -128, 127), m an fp32 product of scales."""
    t = np.asarray(acc, dtype=np.int32).astype(np.float32) * np.float32(m)
    return np.clip(rne(t), QMIN, QMAX).astype(np.int8)


def absmax_scale(X) -> np.float32:
    """s = max|X| / 127 as fp32 (1 when X is all zero, a case the paper does not cover)."""
    X = np.asarray(X)
    m = float(np.max(np.abs(X))) if X.size else 0.0
    return np.float32(m / QMAX) if m > 0.0 else np.float32(1.0)


def percentile_max(X, p: float) -> float:
    """max^p(|X|) of Section 4.2: nearest-rank percentile over all elements of |X| at once:
    the value of 1-based rank ceil(p/100 * n) in ascending order (p = 100 gives the maximum)."""
    a = np.sort(np.abs(np.asarray(X, dtype=np.float64)).ravel())
    n = a.size
    rank = int(math.ceil(float(p) * float(n) / 100.0))
    rank = min(max(rank, 1), n)
    return float(a[rank - 1])


def clip_mse_model(X, s: float, bits: int = 8) -> float:
    """Modelled squared error of quantizing X with clipping scalar s: uniform rounding noise
    s^2 4^-bits / 3 on every nonzero element inside [-s, s] (step 2s / 2^bits, variance
    step^2 / 12), plus the clipping error (|x| - s)^2 of every element outside."""
    a = np.abs(np.asarray(X, dtype=np.float64)).ravel()
    inside = (a > 0.0) & (a <= s)
    outside = a > s
    return float(4.0 ** (-bits) / 3.0 * s * s * np.count_nonzero(inside) + np.sum((a[outside] - s) ** 2))


def optimal_clip(X, bits: int = 8, max_iters: int = 32) -> float:
    """Clipping scalar that minimises `clip_mse_model` (the clipping optimisation named in
    Section 5.1 "Quantization setup" for the enhanced variant; the paper cites the algorithm and
    prints none of it, so this is the cited method's fixed-point form of d(model)/ds = 0):

        s <- sum(|x| : |x| > s) / (4^-bits / 3 * count(0 < |x| <= s) + count(|x| > s))

    started at s = mean|x| and repeated until s stops changing, nothing lies outside s, or
    `max_iters` updates were made.  Returns 0 for an all-zero tensor."""
    a = np.abs(np.asarray(X, dtype=np.float64)).ravel()
    if a.size == 0:
        return 0.0
    c = 4.0 ** (-bits) / 3.0
    s = float(np.sum(a) / a.size)
    for _ in range(max_iters):
        outside = a > s
        n_out = int(np.count_nonzero(outside))
        if n_out == 0:
            break
        n_in = int(np.count_nonzero((a > 0.0) & (a <= s)))
        nxt = float(np.sum(a[outside]) / (c * n_in + n_out))
        if nxt == s:
            break
        s = nxt
    return s


def int_matmul(a_q, w_q) -> np.ndarray:
    """Integer GEMM acc[m, j] = sum_k a_q[m, k] * w_q[j, k] (weights stored [out, in]).

    Evaluated as a float64 matrix product of the integer values, which is exact here
    (|acc| <= K * 128 * 128 < 2^53 for any K this path meets)."""
    a = np.asarray(a_q).astype(np.float64)
    w = np.asarray(w_q).astype(np.float64)
    return np.rint(a @ w.T).astype(np.int32)
