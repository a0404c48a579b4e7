"""Pins for the oracle's conv, selective scan, fp mixer and quantized mixer
(Section 3.1 Eq. 1; Section 4.1 Theorem; Sections 4.2, 4.3; Appendix "Quantization Error
Analysis" unrolled form; Table "quamba_ablation" qualitatively)."""
import numpy as np
import pytest

import oracle as O
import workloads as W


# ------------------------------------------------------------------ conv
def test_conv_equals_toeplitz_product():
    rng = np.random.default_rng(0)
    L, Di, Wd = 9, 3, 4
    x = rng.standard_normal((1, L, Di))
    w = rng.standard_normal((Di, Wd))
    b = rng.standard_normal(Di)
    got = O.causal_conv_fp(x, w, b)
    for d in range(Di):
        T = np.zeros((L, L))
        for t in range(L):
            for s in range(L):
                lag = t - s  # weight index W-1-lag multiplies the sample lag steps back
                if 0 <= lag < Wd:
                    T[t, s] = w[d, Wd - 1 - lag]
        assert np.allclose(got[0, :, d], T @ x[0, :, d] + b[d], atol=1e-12)


def test_conv_causal_and_history():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 12, 5))
    w = rng.standard_normal((5, 4))
    b = np.zeros(5)
    base = O.causal_conv_fp(x, w, b)
    x2 = x.copy()
    x2[:, 7] += 10.0
    pert = O.causal_conv_fp(x2, w, b)
    assert np.array_equal(base[:, :7], pert[:, :7])
    assert not np.allclose(base[:, 7:11], pert[:, 7:11])
    assert np.array_equal(base[:, 11:], pert[:, 11:])  # width 4: reaches 3 steps ahead only
    # splitting the sequence and carrying the last W-1 inputs gives the same result
    tail = O.causal_conv_fp(x[:, 5:], w, b, history=x[:, 2:5])
    assert np.allclose(tail, base[:, 5:], atol=1e-12)


# ------------------------------------------------------------------ scan
def _rand_scan(rng, Bt=2, L=7, Di=3, N=4):
    x = rng.standard_normal((Bt, L, Di))
    dt = rng.uniform(0.01, 0.5, (Bt, L, Di))
    A = -rng.uniform(0.5, 3.0, (Di, N))
    Bm = rng.standard_normal((Bt, L, N))
    Cm = rng.standard_normal((Bt, L, N))
    D = rng.standard_normal(Di)
    z = rng.standard_normal((Bt, L, Di))
    return x, dt, A, Bm, Cm, D, z


def test_scan_reduces_to_cumsum():
    rng = np.random.default_rng(2)
    Bt, L, Di, N = 2, 50, 4, 16
    x = rng.standard_normal((Bt, L, Di))
    dt = np.full((Bt, L, Di), 0.25)
    A = np.zeros((Di, N))
    ones = np.ones((Bt, L, N))
    z = np.full((Bt, L, Di), 50.0)  # SiLU(50) = 50 to 1e-20: the gate is a known constant
    g, y, h = O.selective_scan(x, dt, A, ones, ones, np.zeros(Di), z)
    assert np.allclose(y, 0.25 * N * np.cumsum(x, axis=1), atol=1e-12)
    assert np.allclose(g, y * 50.0, rtol=1e-12)
    assert np.allclose(h, 0.25 * np.cumsum(x, axis=1)[:, -1, :, None] * np.ones(N), atol=1e-12)


def test_scan_unrolled_sum():
    """h_T = sum_s (prod_{u>s} exp(dt_u A)) dt_s B_s x_s, written out term by term."""
    rng = np.random.default_rng(3)
    x, dt, A, Bm, Cm, D, z = _rand_scan(rng, Bt=1, L=6, Di=2, N=3)
    g, y, h = O.selective_scan(x, dt, A, Bm, Cm, D, z)
    for d in range(2):
        for T in range(6):
            acc_y = 0.0
            for n in range(3):
                hn = 0.0
                for s in range(T + 1):
                    decay = 1.0
                    for u in range(s + 1, T + 1):
                        decay *= np.exp(dt[0, u, d] * A[d, n])
                    hn += decay * dt[0, s, d] * Bm[0, s, n] * x[0, s, d]
                acc_y += Cm[0, T, n] * hn
                if T == 5:
                    assert np.isclose(h[0, d, n], hn, rtol=1e-12)
            acc_y += D[d] * x[0, T, d]
            assert np.isclose(y[0, T, d], acc_y, rtol=1e-11, atol=1e-13)
            sig = 1.0 / (1.0 + np.exp(-z[0, T, d]))
            assert np.isclose(g[0, T, d], acc_y * z[0, T, d] * sig, rtol=1e-11, atol=1e-13)


def test_scan_chunk_splitting():
    rng = np.random.default_rng(4)
    x, dt, A, Bm, Cm, D, z = _rand_scan(rng, Bt=2, L=23, Di=5, N=16)
    g, y, h = O.selective_scan(x, dt, A, Bm, Cm, D, z)
    s = 9
    g1, _, h1 = O.selective_scan(x[:, :s], dt[:, :s], A, Bm[:, :s], Cm[:, :s], D, z[:, :s])
    g2, _, h2 = O.selective_scan(x[:, s:], dt[:, s:], A, Bm[:, s:], Cm[:, s:], D, z[:, s:], h0=h1)
    assert np.allclose(np.concatenate([g1, g2], axis=1), g, rtol=1e-12, atol=1e-14)
    assert np.allclose(h2, h, rtol=1e-12, atol=1e-14)


def test_scan_frozen_and_forgetful_limits():
    rng = np.random.default_rng(5)
    x, dt, A, Bm, Cm, D, z = _rand_scan(rng, Bt=1, L=5, Di=3, N=4)
    h0 = rng.standard_normal((1, 3, 4))
    # dt -> 0 (very negative pre-softplus): the state does not move
    tiny = np.full_like(dt, float(O.softplus(np.array(-60.0))))
    _, _, h = O.selective_scan(x, tiny, A, Bm, Cm, D, z, h0=h0)
    assert np.allclose(h, h0, atol=1e-20, rtol=1e-12)
    # dt large: the old state is forgotten, h_t = dt B_t x_t
    big = np.full_like(dt, 200.0)
    _, _, h = O.selective_scan(x, big, A, Bm, Cm, D, z, h0=h0)
    assert np.allclose(h[0], 200.0 * x[0, -1, :, None] * Bm[0, -1, None, :], rtol=1e-12)


def test_softplus_silu_values():
    assert np.isclose(O.softplus(np.array(0.0)), np.log(2.0))
    assert O.softplus(np.array(30.0)) == 30.0
    assert np.isclose(O.softplus(np.array(-30.0)), np.exp(-30.0), rtol=1e-9)
    assert np.isclose(O.silu(np.array(0.0)), 0.0)
    assert np.isclose(O.silu(np.array(1.0)), 1.0 / (1.0 + np.exp(-1.0)))
    assert np.isclose(O.silu(np.array(-1.0)), -1.0 / (1.0 + np.e))


def test_theorem_lti_error_bound():
    """Theorem 4.1 (time-invariant corollary): with ||A_bar|| <= a < 1, ||B_bar|| <= b and input
    perturbations of norm <= eps, ||h_bar(T) - h(T)|| <= eps b / (1 - a)."""
    rng = np.random.default_rng(6)
    L, N, dt0 = 400, 16, 0.1
    a_n = rng.uniform(0.2, 0.9, N)
    a = a_n.max()
    A = (np.log(a_n) / dt0)[None, :]                      # exp(dt A) = a_n
    Bvec = rng.standard_normal(N)
    b = dt0 * np.linalg.norm(Bvec)                        # B_bar = dt * B
    eps = 0.03
    x = rng.standard_normal((1, L, 1))
    delta = rng.uniform(-eps, eps, (1, L, 1))
    delta[0, -50:, 0] = eps * np.sign(Bvec[np.argmax(a_n)])  # push towards the worst case
    dt = np.full((1, L, 1), dt0)
    Bm = np.tile(Bvec, (1, L, 1))
    z = np.zeros((1, L, 1))
    _, _, h = O.selective_scan(x, dt, A, Bm, Bm, np.zeros(1), z)
    _, _, hq = O.selective_scan(x + delta, dt, A, Bm, Bm, np.zeros(1), z)
    err = np.linalg.norm(hq - h)
    assert err <= eps * b / (1 - a)
    assert err > 0.05 * eps * b / (1 - a)  # the bound is not vacuous for this instance


# ------------------------------------------------------------------ fp mixer
def test_fp_forward_lti_closed_form():
    """Constant input and a conv history equal to it make x, dt, B, C constant in time, so
    h_t = dt B x (1 - a^t) / (1 - a) with a = exp(dt A): a geometric series."""
    cfg = W.tiny_config(d_model=16, d_inner=32, dt_rank=4, batch=1, seqlen=11)
    w = W.make_weights(cfg, randomize_bias=True)
    for k in ("W_in", "conv_w", "W_x", "W_dt", "W_out"):
        w[k] = w[k] * 20.0  # make every stage contribute visibly
    rng = np.random.default_rng(7)
    u0 = rng.standard_normal(cfg.d_model)
    u = np.tile(u0, (1, cfg.seqlen, 1))
    Di, R, N = cfg.d_inner, cfg.dt_rank, cfg.d_state
    f = lambda k: w[k].astype(np.float64)  # noqa: E731
    xz = f("W_in") @ u0
    hist = np.tile(xz[:Di], (1, 3, 1))
    t = O.fp_forward(w, u, conv_history=hist)
    xc = f("conv_b") + f("conv_w").sum(axis=1) * xz[:Di]
    x = xc / (1 + np.exp(-xc))
    dbc = f("W_x") @ x
    dt = np.log1p(np.exp(f("W_dt") @ dbc[:R] + f("dt_bias")))
    A = -np.exp(f("A_log"))
    a = np.exp(dt[:, None] * A)
    zc = xz[Di:]
    for step in (1, 2, 5, 11):
        h = (dt * x)[:, None] * dbc[None, R:R + N] * (1 - a ** step) / (1 - a)
        y = h @ dbc[R + N:] + f("D") * x
        out = f("W_out") @ (y * zc / (1 + np.exp(-zc)))
        assert np.allclose(t["out"][0, step - 1], out, rtol=1e-9, atol=1e-12)
    assert np.allclose(t["h"][0], h, rtol=1e-9)


def test_fp_forward_split_orders():
    """Rows [0,Di) of W_in feed the conv/scan branch and rows [Di,2Di) the gate; rows of W_x
    are dt | B | C: zeroing a block must have exactly the effect the wiring implies."""
    cfg = W.tiny_config(d_model=16, d_inner=32, dt_rank=4, batch=1, seqlen=6)
    w = W.make_weights(cfg, randomize_bias=True)
    for k in ("W_in", "conv_w", "W_x", "W_dt", "W_out"):
        w[k] = w[k] * 20.0
    u = W.make_hidden(cfg)
    Di, R, N = cfg.d_inner, cfg.dt_rank, cfg.d_state
    wz = dict(w); wz["W_in"] = w["W_in"].copy(); wz["W_in"][Di:] = 0   # gate branch off -> SiLU(0)=0
    assert np.all(O.fp_forward(wz, u)["out"] == 0)
    wc = dict(w); wc["W_x"] = w["W_x"].copy(); wc["W_x"][R + N:] = 0    # C = 0 -> y = D x
    t = O.fp_forward(wc, u)
    assert np.allclose(t["y"], w["D"].astype(np.float64) * t["x"], rtol=1e-12)
    wb = dict(w); wb["W_x"] = w["W_x"].copy(); wb["W_x"][R:R + N] = 0   # B = 0 -> state stays 0
    assert np.all(O.fp_forward(wb, u)["h"] == 0)
    wd = dict(w); wd["W_x"] = w["W_x"].copy(); wd["W_x"][:R] = 0        # dt_low = 0 -> dt = softplus(bias)
    t = O.fp_forward(wd, u)
    assert np.allclose(t["dt"], np.log1p(np.exp(w["dt_bias"].astype(np.float64))), rtol=1e-12)


# ------------------------------------------------------------------ quantized mixer
@pytest.fixture(scope="module")
def tiny_setup():
    cfg = W.tiny_config(d_model=64, d_inner=128, dt_rank=16, batch=2, seqlen=40, n_outlier=0)
    w = W.make_weights(cfg, randomize_bias=True)
    for k in ("W_in", "conv_w", "W_x", "W_dt", "W_out"):
        w[k] = w[k] * 10.0
    calib = W.make_calibration(cfg)
    qw, sc = O.calibrate(w, calib, 100.0)
    return cfg, w, calib, qw, sc


def test_calibrate_scales_and_weights(tiny_setup):
    cfg, w, calib, qw, sc = tiny_setup
    t = O.fp_forward(w, calib)
    assert np.isclose(float(sc["s_xpre"]) * 127, np.abs(t["x_pre"]).max(), rtol=1e-6)
    assert np.isclose(float(sc["s_dt"]) * 127, np.abs(t["dt_raw"]).max(), rtol=1e-6)
    assert np.isclose(float(sc["s_A"]) * 127, 16.0, rtol=1e-6)
    assert all(v.dtype == np.float32 for v in sc.values())
    for k in ("W_in", "conv_w", "W_x", "W_dt", "A", "D", "W_outH"):
        assert qw[k].dtype == np.int8 and np.abs(qw[k].astype(int)).max() == 127
    assert qw["A"].max() <= 0
    # dequantized folded weight reproduces W_out through the inverse transform
    H = O.hadamard_matrix(cfg.d_inner).astype(np.float64)
    back = (float(sc["s_WoutH"]) * qw["W_outH"].astype(np.float64)) @ H / cfg.d_inner
    assert np.abs(back - w["W_out"]).max() <= float(sc["s_WoutH"])  # << 1 LSB after averaging
    # multipliers are the stated products
    assert np.isclose(float(sc["m_out"]), float(sc["s_y"]) * float(sc["s_WoutH"]) / cfg.d_inner, rtol=1e-6)
    assert np.isclose(float(sc["m_in_z"]), float(sc["s_u"]) * float(sc["s_Win"]) / float(sc["s_z"]), rtol=1e-6)
    assert np.isclose(float(sc["m_dt"]), float(sc["s_dtl"]) * float(sc["s_Wdt"]) / float(sc["s_dt"]), rtol=1e-6)


def test_quantized_tracks_fp(tiny_setup):
    cfg, w, calib, qw, sc = tiny_setup
    u = calib  # inside the calibrated range: nothing saturates, errors are rounding only
    r = O.q_prefill(qw, sc, u)
    ref = O.fp_forward(w, u)
    for name, got, want in [
        ("x_pre", float(sc["s_xpre"]) * r["xpre_q"], ref["x_pre"]),
        ("z", float(sc["s_z"]) * r["z_q"], ref["z"]),
        ("x", float(sc["s_x"]) * r["x_q"], ref["x"]),
        ("B", float(sc["s_B"]) * r["B_q"], ref["B"]),
        ("C", float(sc["s_C"]) * r["C_q"], ref["C"]),
        ("dt_raw", float(sc["s_dt"]) * r["dt_q"], ref["dt_raw"]),
        ("g", r["g"], ref["g"]),
        ("gH", float(sc["s_y"]) * r["gH_q"], ref["g"] @ O.hadamard_matrix(cfg.d_inner).astype(float).T),
        ("out", r["out"].astype(np.float64), ref["out"]),
    ]:
        err = np.abs(got - want).max() / np.abs(want).max()
        assert err < 0.05, (name, err)
    assert r["out"].dtype == np.float16 and r["g16"].dtype == np.float16
    assert r["h"].dtype == np.float32 and r["conv_state"].dtype == np.float16
    assert np.abs(r["h"] - ref["h"]).max() / np.abs(ref["h"]).max() < 0.05


def test_prefill_then_decode_matches_longer_prefill(tiny_setup):
    cfg, w, calib, qw, sc = tiny_setup
    u = W.make_hidden(cfg, seqlen=cfg.seqlen + 3)
    full = O.q_prefill(qw, sc, u)
    part = O.q_prefill(qw, sc, u[:, :cfg.seqlen])
    h, cs = part["h"], part["conv_state"]
    for i in range(3):
        d = O.q_decode(qw, sc, u[:, cfg.seqlen + i], h, cs)
        h, cs = d["h"], d["conv_state"]
        diff = np.abs(d["x_q"][:, 0].astype(int) - full["x_q"][:, cfg.seqlen + i].astype(int))
        assert diff.max() <= 1 and (diff > 0).mean() <= 0.01
        ref = full["out"][:, cfg.seqlen + i].astype(np.float64)
        assert np.abs(d["out"][:, 0].astype(np.float64) - ref).max() <= 0.05 * np.abs(ref).max()
    assert np.abs(h - full["h"]).max() <= 0.02 * np.abs(full["h"]).max()
    assert np.array_equal(cs, full["conv_state"])


def test_prefill_carries_initial_state(tiny_setup):
    cfg, w, calib, qw, sc = tiny_setup
    u = W.make_hidden(cfg)
    rng = np.random.default_rng(3)
    h0 = rng.standard_normal((cfg.batch, cfg.d_inner, cfg.d_state)).astype(np.float32)
    a = O.q_prefill(qw, sc, u)
    b = O.q_prefill(qw, sc, u, h0=h0)
    assert np.array_equal(a["dt_q"], b["dt_q"])
    assert not np.allclose(a["g"], b["g"])


def test_hadamard_and_percentile_help_with_outliers():
    """Qualitative content of Table "quamba_ablation": with large outliers in the scan output
    the Hadamard-space quantization of y has far lower error than quantizing y directly; with
    rare outliers in x the percentile scale lowers the error of typical values."""
    rng = np.random.default_rng(11)
    n = 1536
    y = rng.standard_normal((64, n))
    y[:, 17] *= 300.0
    H = O.hadamard_matrix(n).astype(np.float64)
    s_direct = O.absmax_scale(y)
    yq = float(s_direct) * O.quantize(y.astype(np.float32), np.float32(1 / float(s_direct))).astype(np.float64)
    yH = y @ H.T
    s_h = O.absmax_scale(yH)
    yHq = float(s_h) * O.quantize(yH.astype(np.float32), np.float32(1 / float(s_h))).astype(np.float64)
    back = yHq @ H / n
    mask = np.ones(n, bool); mask[17] = False
    e_direct = np.abs(yq - y)[:, mask].mean()
    e_had = np.abs(back - y)[:, mask].mean()
    assert e_had < 0.2 * e_direct
    x = np.abs(rng.standard_normal(200000)) * 0.3
    x[:20] = 9.0  # 0.01 % outliers
    s_max = np.float32(O.percentile_max(x, 100.0) / 127)
    s_p = np.float32(O.percentile_max(x, 99.9) / 127)
    body = x[20:].astype(np.float32)
    e_max = np.abs(float(s_max) * O.quantize(body, np.float32(1 / float(s_max))) - body).mean()
    e_p = np.abs(float(s_p) * O.quantize(body, np.float32(1 / float(s_p))) - body).mean()
    assert e_p < 0.25 * e_max


def test_add_rmsnorm_quant():
    rng = np.random.default_rng(12)
    a = rng.standard_normal((5, 64)).astype(np.float16)
    r = rng.standard_normal((5, 64)).astype(np.float16)
    wt = np.ones(64, dtype=np.float16)
    q, res = O.add_rmsnorm_quant(a, r, wt, np.float32(127.0 / 4.0), eps=0.0)
    assert res.dtype == np.float16 and q.dtype == np.int8
    assert np.array_equal(res, (a.astype(np.float32) + r.astype(np.float32)).astype(np.float16))
    # unit-RMS rows: dequantized values have mean square 1 up to quantization error
    dq = q.astype(np.float64) * 4.0 / 127.0
    assert np.allclose((dq ** 2).mean(axis=-1), 1.0, atol=0.02)
    # scaling the input leaves the normalised output unchanged
    q2, _ = O.add_rmsnorm_quant((a.astype(np.float32) * 4).astype(np.float16),
                                (r.astype(np.float32) * 4).astype(np.float16), wt,
                                np.float32(127.0 / 4.0), eps=0.0)
    assert np.abs(q2.astype(int) - q.astype(int)).max() <= 1


def test_add_rmsnorm_quant_closed_form_places_weight_and_eps():
    """Section 4.3 "Fused RMSNorm", written out for rows whose sum is a constant c: RMSNorm gives
    w_j c / sqrt(c^2 + eps) in column j, so the codes are q(w_j c / sqrt(c^2 + eps) / s).  A graded
    weight pins the weight multiply (position and per-column use); a small c makes eps matter: with
    c^2 = eps the factor is 1/sqrt(2), with eps outside the root it would be 1/(1 + sqrt(eps)/|c|) = 1/2,
    without eps 1."""
    Dm = 64
    w = np.linspace(0.5, 1.5, Dm).astype(np.float16)
    inv_s = np.float32(127.0 / 2.0)
    # |c| = 3: eps is negligible, the weight is not
    half = np.full((2, Dm), 1.5, dtype=np.float16)
    half[1] = -1.5
    q, res = O.add_rmsnorm_quant(half, half, w, inv_s, eps=1e-5)
    assert np.array_equal(res, (half * 2).astype(np.float16))
    y = w.astype(np.float64) * 3.0 / np.sqrt(9.0 + 1e-5)
    want = np.clip(np.rint((y.astype(np.float32) * inv_s)), -128, 127).astype(np.int8)
    assert np.array_equal(q[0], want) and np.array_equal(q[1], -want)
    assert len(np.unique(q[0])) > 30  # the weight really grades the row
    # c^2 = eps exactly (c = 2^-6, eps = 2^-12): the three placements of eps give three different rows
    c, eps = 2.0 ** -6, 2.0 ** -12
    a = np.full((1, Dm), c, dtype=np.float16)
    q, res = O.add_rmsnorm_quant(a, np.zeros_like(a), w, inv_s, eps=eps)
    inside = np.rint((w.astype(np.float64) / np.sqrt(2.0)).astype(np.float32) * inv_s).astype(np.int8)
    outside = np.rint((w.astype(np.float64) / 2.0).astype(np.float32) * inv_s).astype(np.int8)
    absent = np.rint(w.astype(np.float32) * inv_s).astype(np.int8)
    assert np.array_equal(q[0], inside)
    assert not np.array_equal(inside, outside) and not np.array_equal(inside, absent)
    # a non-constant row against the definition written out element by element in plain Python
    rng = np.random.default_rng(3)
    xo = rng.standard_normal((1, 8)).astype(np.float16)
    xr = rng.standard_normal((1, 8)).astype(np.float16)
    w8 = np.linspace(0.25, 2.0, 8).astype(np.float16)
    q, res = O.add_rmsnorm_quant(xo, xr, w8, np.float32(127.0 / 6.0), eps=1e-5)
    ssum = [float(np.float16(np.float32(xo[0, j]) + np.float32(xr[0, j]))) for j in range(8)]
    ms = sum(v * v for v in ssum) / 8.0
    for j in range(8):
        yj = np.float32(ssum[j] / (ms + 1e-5) ** 0.5 * float(w8[j]))
        assert q[0, j] == int(np.clip(np.rint(yj * np.float32(127.0 / 6.0)), -128, 127))
