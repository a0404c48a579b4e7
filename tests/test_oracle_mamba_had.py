"""Pins for the oracle's Appendix H comparison variant (rotation on the scan-input path)."""
import dataclasses

import numpy as np
import pytest

import oracle as O
import workloads as W


@pytest.mark.parametrize("n", [64, 192, 320, 1536])
def test_transform_pair_returns_its_input(n):
    """(1/n) H^T (H v) = v, in the row forms the oracle uses (v @ H.T forward, v @ H backward).
    For the Paley factors H is not symmetric: going forward twice does not return v."""
    H = O.hadamard_matrix(n).astype(np.float64)
    rng = np.random.default_rng(n)
    v = rng.integers(-100, 100, size=(3, n)).astype(np.float64)
    assert np.array_equal((v @ H.T) @ H / n, v)
    if O.hadamard_factor(n)[0] > 1:
        assert not np.array_equal((v @ H.T) @ H.T / n, v)
    q = rng.integers(-128, 128, size=(2, n)).astype(np.int8)
    want = (np.float32(0.01) * (q.astype(np.float64) @ H).astype(np.float32)).astype(np.float16)
    assert np.array_equal(O.hadamard_inverse_dequant(q, 0.01).view(np.uint16), want.view(np.uint16))


def _setup(x_rows=0, gain=1.0, outlier_gain=None, **kw):
    cfg = W.tiny_config(name="th", d_model=64, d_inner=192, dt_rank=16, config_id=97, **kw)
    if outlier_gain is not None:
        cfg = dataclasses.replace(cfg, outlier_gain=outlier_gain)
    w = W.make_weights(cfg, randomize_bias=True, x_outlier_rows=x_rows, x_outlier_gain=gain)
    return cfg, w, W.make_calibration(cfg)


def test_folded_x_proj_weight_reproduces_the_projection():
    """(H w_r) . (H x) / n = w_r . x for every row of W_x (the fold into the linear layer)."""
    cfg, w, calib = _setup()
    _, _, hx = O.calibrate_hadx(w, calib)
    Di = cfg.d_inner
    H = O.hadamard_matrix(Di).astype(np.float64)
    x = np.random.default_rng(3).standard_normal((5, Di))
    assert np.allclose((x @ H.T) @ hx["W_xH_fp"].T / Di, x @ np.asarray(w["W_x"], np.float64).T, rtol=0, atol=1e-12)
    # the int8 weight and its scale describe that matrix
    assert np.abs(hx["W_xH"].astype(np.float64) * float(hx["s_WxH"]) - hx["W_xH_fp"]).max() <= float(hx["s_WxH"]) / 2 * 1.0001
    assert float(hx["xhat_scale"]) == pytest.approx(float(hx["s_xH"]) / Di, rel=1e-6)


def test_reconstruction_error_is_what_the_quantizer_implies():
    """x_hat - x16 = (1/n) H^T e with |e_i| <= s_xH / 2 (no clipping on the calibration data):
    its L2 norm per row is at most s_xH / 2 (H^T / sqrt(n) is orthogonal), plus half-precision rounding."""
    cfg, w, calib = _setup()
    qw, sc, hx = O.calibrate_hadx(w, calib)
    t = O.q_prefill_hadx(qw, sc, hx, calib)
    err = t["xhat16"].astype(np.float64) - t["x16"].astype(np.float64)
    bound = float(hx["s_xH"]) / 2 + 2.0 ** -11 * np.linalg.norm(t["x16"].astype(np.float64), axis=-1).max()
    assert np.linalg.norm(err, axis=-1).max() <= bound
    assert np.linalg.norm(err, axis=-1).max() >= 0.1 * float(hx["s_xH"]) / 2  # and it is not trivially zero


def test_variant_tracks_the_unquantized_mixer_on_par_with_quamba():
    """Section 5.1 / Appendix H: the variant is on par with Quamba in accuracy.  Checked as error
    against the unquantized mixer, also with far-reaching scan-input channels; the error of the x
    path alone is compared with plain rounding of x on the absmax grid, which it must not exceed
    by more than the spread of the two grids explains."""
    for rows, gain in ((0, 1.0), (4, 8.0)):
        cfg, w, calib = _setup(x_rows=rows, gain=gain, outlier_gain=1.0)
        u = W.make_hidden(cfg, batch=2, seqlen=48, stream=7)
        ref = O.fp_forward(w, u)["out"]
        rel = lambda out: np.linalg.norm(out.astype(np.float64) - ref) / np.linalg.norm(ref)  # noqa: E731
        qw, sc, hx = O.calibrate_hadx(w, calib)
        t = O.q_prefill_hadx(qw, sc, hx, u)
        e_had, e_quamba = rel(t["out"]), rel(O.q_prefill(qw, sc, u)["out"])
        assert e_had < 0.12 and abs(e_had - e_quamba) < 0.1 * e_quamba, (rows, e_had, e_quamba)
        x = t["x16"].astype(np.float64)
        rms_had = np.sqrt(np.mean((t["xhat16"].astype(np.float64) - x) ** 2))
        # uniform rounding noise of the rotated grid, carried back: s_xH / sqrt(12 n)
        assert rms_had == pytest.approx(float(hx["s_xH"]) / np.sqrt(12.0 * cfg.d_inner), rel=0.15)


def test_decode_continues_prefill():
    cfg, w, calib = _setup()
    qw, sc, hx = O.calibrate_hadx(w, calib)
    u = W.make_hidden(cfg, batch=2, seqlen=21, stream=9)
    full = O.q_prefill_hadx(qw, sc, hx, u)
    part = O.q_prefill_hadx(qw, sc, hx, u[:, :20])
    step = O.q_decode_hadx(qw, sc, hx, u[:, 20], part["h"], part["conv_state"])
    a, b = step["out"][:, 0].astype(np.float64), full["out"][:, 20].astype(np.float64)
    assert np.abs(a - b).max() <= 2e-2 * np.abs(b).max()
    assert np.abs(step["h"] - full["h"]).max() <= 2e-2 * np.abs(full["h"]).max()
    assert np.array_equal(step["conv_state"].view(np.uint16), full["conv_state"].view(np.uint16))
