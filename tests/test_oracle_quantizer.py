"""Pins for the oracle's quantizer, percentile and integer GEMM (Section 3.2 Eq. 2;
Section 4.2 percentile maximum)."""
import numpy as np
import pytest

from oracle import absmax_scale, int_matmul, percentile_max, quantize, requant_acc


def test_ties_to_even_and_clamp():
    v = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, 127.5, 300.0, -128.5, -129.0, -1e9],
                 dtype=np.float32)
    q = quantize(v, 1.0)
    assert q.dtype == np.int8
    assert q.tolist() == [0, 2, 2, 0, -2, -2, 126, 127, 127, -128, -128, -128]


def test_scale_maps_absmax_to_127():
    rng = np.random.default_rng(0)
    X = rng.standard_normal(10000).astype(np.float32) * 3
    s = absmax_scale(X)
    assert s.dtype == np.float32
    assert np.isclose(float(s) * 127, np.abs(X).max(), rtol=1e-6)
    q = quantize(X, np.float32(1.0 / float(s)))
    assert q[np.argmax(np.abs(X))] in (127, -127)
    assert q.min() >= -127  # -128 is reachable only by clipped values
    assert absmax_scale(np.zeros(4)) == np.float32(1.0)


def test_roundtrip_error_bound_and_saturation():
    rng = np.random.default_rng(1)
    s = np.float32(0.037)
    inv = np.float32(1.0 / float(s))
    X = (rng.uniform(-127, 127, 200000) * float(s)).astype(np.float32)
    q = quantize(X, inv)
    err = np.abs(X.astype(np.float64) - float(s) * q.astype(np.float64))
    assert err.max() <= float(s) / 2 * (1 + 1e-5)
    big = np.array([200 * s, -200 * s, 127.4 * s, -128.6 * s], dtype=np.float32)
    assert quantize(big, inv).tolist() == [127, -128, 127, -128]


def test_idempotent():
    rng = np.random.default_rng(2)
    s = np.float32(0.0123)
    inv = np.float32(1.0 / float(s))
    X = rng.standard_normal(50000).astype(np.float32)
    q = quantize(X, inv)
    again = quantize((s * q.astype(np.float32)).astype(np.float32), inv)
    assert np.array_equal(q, again)


def test_requant_acc_is_one_multiply():
    acc = np.array([0, 1, -1, 1000, -1000, 2**24 + 1, -(2**30)], dtype=np.int32)
    m = np.float32(0.0125)
    want = np.clip(np.rint(acc.astype(np.float32) * m), -128, 127).astype(np.int8)
    assert np.array_equal(requant_acc(acc, m), want)
    assert requant_acc(np.array([40, 120], dtype=np.int32), np.float32(0.0125)).tolist() == [0, 2]


@pytest.mark.parametrize("n,p", [(10, 50.0), (10, 90.0), (10, 91.0), (1000, 99.9), (1000, 99.999),
                                 (12345, 99.0), (7, 100.0), (7, 0.0)])
def test_percentile_nearest_rank(n, p):
    rng = np.random.default_rng(n)
    X = rng.standard_normal(n)
    a = sorted(abs(v) for v in X)
    # brute force: smallest value v such that at least p% of the elements are <= v
    need = p / 100.0 * n
    want = next((v for i, v in enumerate(a) if i + 1 >= need - 1e-9), a[-1])
    if p == 0.0:
        want = a[0]
    assert percentile_max(X, p) == want


def test_percentile_limits_and_monotone():
    rng = np.random.default_rng(5)
    X = rng.standard_normal((4, 300, 20))
    assert percentile_max(X, 100.0) == np.abs(X).max()
    ps = [50, 90, 99, 99.9, 99.99, 99.999, 100]
    vals = [percentile_max(X, p) for p in ps]
    assert all(a <= b for a, b in zip(vals, vals[1:]))
    X2 = X.copy()
    X2.ravel()[::4001] *= 1000  # a handful of outliers moves the max but not p=99.9
    assert percentile_max(X2, 100.0) > 100 * percentile_max(X2, 99.9)
    assert abs(percentile_max(X2, 99.0) - percentile_max(X, 99.0)) < 0.05


@pytest.mark.parametrize("M,N,K", [(3, 5, 7), (8, 4, 48), (5, 9, 160)])
def test_int_matmul_vs_loops(M, N, K):
    rng = np.random.default_rng(M * 100 + N)
    a = rng.integers(-128, 128, (M, K), dtype=np.int8)
    w = rng.integers(-128, 128, (N, K), dtype=np.int8)
    want = np.zeros((M, N), dtype=np.int64)
    for i in range(M):
        for j in range(N):
            s = 0
            for k in range(K):
                s += int(a[i, k]) * int(w[j, k])
            want[i, j] = s
    got = int_matmul(a, w)
    assert got.dtype == np.int32
    assert np.array_equal(got.astype(np.int64), want)


def test_int_matmul_extreme_values_exact():
    K = 8192
    a = np.full((2, K), -128, dtype=np.int8)
    w = np.full((3, K), -128, dtype=np.int8)
    assert np.all(int_matmul(a, w) == K * 128 * 128)
    w[1] = 127
    assert np.all(int_matmul(a, w)[:, 1] == -K * 128 * 127)
    rng = np.random.default_rng(9)
    a = rng.integers(-128, 128, (64, K), dtype=np.int8)
    w = rng.integers(-128, 128, (32, K), dtype=np.int8)
    assert np.array_equal(int_matmul(a, w).astype(np.int64), a.astype(np.int64) @ w.astype(np.int64).T)


# ---------------------------------------------------------------- optimal clipping scalar
def _heavy_tailed(seed, n=60000, n_big=40, gain=9.0):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(n)
    x[rng.choice(n, n_big, replace=False)] *= gain
    return x.astype(np.float32)


def test_clip_model_matches_measured_rounding_and_clipping_error():
    """The noise model behind the clipping optimisation (Section 5.1, enhanced variant): rounding
    noise of a 2^bits-level grid over [-s, s] plus the squared overshoot of clipped values,
    against the error of actually rounding and clipping."""
    from oracle import clip_mse_model
    rng = np.random.default_rng(5)
    for bits, s in ((8, 2.0), (6, 3.5), (4, 1.0)):
        x = rng.uniform(-1.4 * s, 1.4 * s, 400000)
        step = 2.0 * s / 2 ** bits
        xq = np.clip(np.rint(x / step) * step, -s, s)
        measured = float(np.sum((x - xq) ** 2))
        assert clip_mse_model(x, s, bits) == pytest.approx(measured, rel=0.02)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_optimal_clip_minimises_the_model(seed):
    from oracle import clip_mse_model, optimal_clip
    x = _heavy_tailed(seed)
    s = optimal_clip(x)
    a = np.abs(x.astype(np.float64))
    assert a.mean() < s < a.max()
    grid = np.linspace(0.05 * a.max(), a.max(), 3000)
    j = np.array([clip_mse_model(x, g) for g in grid])
    best = grid[np.argmin(j)]
    assert abs(s - best) <= 2 * (grid[1] - grid[0])
    assert clip_mse_model(x, s) <= j.min() * (1 + 1e-9)
    # every percentile of the paper's sweep (Table "percentiles") is a clip the model rates no better
    for p in (99.0, 99.9, 99.99, 99.999, 100.0):
        assert clip_mse_model(x, s) <= clip_mse_model(x, percentile_max(x, p)) * (1 + 1e-9)


def test_optimal_clip_two_level_closed_form():
    """n_in values of magnitude 1 and one value of magnitude M: the stationary point is
    M / (4^-bits / 3 * n_in + 1), reached from the mean in a few updates."""
    from oracle import optimal_clip
    n_in, M = 1000, 100.0
    x = np.concatenate([np.ones(n_in), [-M]])
    for bits in (8, 4):
        c = 4.0 ** (-bits) / 3.0
        assert optimal_clip(x, bits=bits) == pytest.approx(M / (c * n_in + 1.0), rel=1e-12)


def test_optimal_clip_degenerate_inputs():
    from oracle import optimal_clip
    assert optimal_clip(np.zeros(17)) == 0.0
    assert optimal_clip(np.array([])) == 0.0
    assert optimal_clip(np.full(33, -2.5)) == 2.5       # nothing lies outside the mean
    x = _heavy_tailed(3)
    assert optimal_clip(x, max_iters=64) == optimal_clip(x, max_iters=32)  # converged well before


def test_calibrate_with_optimal_clip_changes_only_the_x_scale():
    from oracle import calibrate, fp_forward, optimal_clip
    import workloads
    cfg = workloads.tiny_config()
    w = workloads.make_weights(cfg)
    cu = workloads.make_calibration(cfg)
    _, sp = calibrate(w, cu)
    _, sm = calibrate(w, cu, x_clip="mse")
    x = fp_forward(w, cu)["x"]
    assert float(sm["s_x"]) == pytest.approx(optimal_clip(np.asarray(x, np.float64).astype(np.float32)) / 127.0, rel=1e-6)
    for k in sp:
        if k in ("s_x", "inv_s_x", "m_x_dt", "m_x_B", "m_x_C"):
            assert sp[k] != sm[k]
        else:
            assert sp[k] == sm[k]
    with pytest.raises(ValueError):
        calibrate(w, cu, x_clip="other")
