"""Pins for the oracle's asymmetric scan-input quantizer (Appendix K, "MinMax Asym. Per.")."""
import dataclasses

import numpy as np
import pytest

import oracle as O
import workloads as W


def _setup(outlier_gain=None, **kw):
    cfg = W.tiny_config(name="ta", d_model=64, d_inner=192, dt_rank=16, config_id=96, **kw)
    if outlier_gain is not None:
        cfg = dataclasses.replace(cfg, outlier_gain=outlier_gain)
    w = W.make_weights(cfg, randomize_bias=True)
    return cfg, w, W.make_calibration(cfg)


def test_affine_quantizer_round_trip_and_range():
    """Inside [lo, hi] the code reproduces the value within half a step; lo and hi land on the two
    ends of the code range; values outside clip."""
    lo, hi = -0.2785, 7.3
    s = np.float32((hi - lo) / 255.0)
    zp = int(np.clip(np.rint(-128.0 - lo / float(s)), -128, 127))
    inv = np.float32(1.0 / float(s))
    x = np.linspace(lo, hi, 20001).astype(np.float32)
    q = O.quantize_asym(x, inv, zp)
    back = float(s) * (q.astype(np.float64) - zp)
    assert np.abs(back - x).max() <= float(s) / 2 * 1.001
    assert q.min() == -128 and q.max() in (126, 127)
    assert O.quantize_asym(np.array([hi * 3, lo * 30], np.float32), inv, zp).tolist() == [127, -128]
    # zero maps to the zero point exactly, so a zero input stays zero after the round trip
    assert O.quantize_asym(np.zeros(1, np.float32), inv, zp)[0] == zp
    # the rounding acts on the shifted value: 3.5, 4.5, 5.5 go to the even neighbour
    assert O.quantize_asym(np.array([0.5, 1.5, 2.5], np.float32), 1.0, 3).tolist() == [4, 4, 6]


def test_column_correction_equals_product_of_shifted_codes():
    """acc[n] - zp * rowsum(W_q[n, :]) = sum_k W_q[n, k] (x_q[k] - zp), by brute force."""
    rng = np.random.default_rng(0)
    xq = rng.integers(-128, 128, size=(7, 96)).astype(np.int8)
    Wq = rng.integers(-128, 128, size=(11, 96)).astype(np.int8)
    for zp in (-128, -119, 0, 5, 127):
        brute = np.zeros((7, 11), dtype=np.int64)
        for m in range(7):
            for n in range(11):
                brute[m, n] = sum(int(Wq[n, k]) * (int(xq[m, k]) - zp) for k in range(96))
        bias = -zp * Wq.astype(np.int64).sum(axis=1)
        assert np.array_equal(O.int_matmul(xq, Wq).astype(np.int64) + bias, brute)


def test_calibrated_grid_is_finer_than_the_symmetric_one():
    """x = SiLU(.) is bounded below by -0.2785 and reaches further above: the asymmetric grid spends
    its 256 levels on [lo, hi] instead of [-hi, hi] (Appendix K: better use of the bit-width), a
    step (127 / 255) (1 - lo / hi) times the symmetric one: one half for far-reaching x."""
    cfg, w, calib = _setup()
    qw, sc, xa = O.calibrate_xasym(w, calib)
    x = O.fp_forward(w, calib)["x"]
    assert -0.2786 <= x.min() < 0
    ratio = float(xa["s_x"]) / float(sc["s_x"])
    lo, hi = float(x.min()), float(sc["s_x"]) * 127
    assert ratio == pytest.approx(127.0 / 255.0 * (1.0 - lo / hi), rel=1e-5) and ratio < 0.85
    assert xa["zero_point"] == int(np.rint(-128.0 - lo / float(xa["s_x"])))
    # both ends of the range are hit on the calibration data itself
    q = O.quantize_asym(np.asarray(x, np.float32), xa["inv_s_x"], xa["zero_point"])
    assert q.min() == -128 and q.max() == 127
    assert np.array_equal(xa["col_bias"], (-xa["zero_point"] * qw["W_x"].astype(np.int64).sum(axis=1)).astype(np.int32))


def test_error_against_the_unquantized_mixer_not_above_quambas():
    cfg, w, calib = _setup(outlier_gain=1.0)
    u = W.make_hidden(cfg, batch=2, seqlen=48, stream=7)
    ref = O.fp_forward(w, u)
    qw, sc, xa = O.calibrate_xasym(w, calib)
    t = O.q_prefill_xasym(qw, sc, xa, u)
    tq = O.q_prefill(qw, sc, u)
    rel = lambda a, b: np.linalg.norm(np.asarray(a, np.float64) - b) / np.linalg.norm(b)  # noqa: E731
    # the x codes themselves: the rounding error shrinks with the step
    e_asym = rel(t["x_deq"], ref["x"])
    e_sym = rel(float(sc["s_x"]) * tq["x_q"].astype(np.float64), ref["x"])
    assert e_asym / e_sym == pytest.approx(float(xa["s_x"]) / float(sc["s_x"]), rel=0.15)
    assert rel(t["out"], ref["out"]) <= 1.02 * rel(tq["out"], ref["out"])


def test_decode_continues_prefill():
    cfg, w, calib = _setup()
    qw, sc, xa = O.calibrate_xasym(w, calib)
    u = W.make_hidden(cfg, batch=2, seqlen=21, stream=9)
    full = O.q_prefill_xasym(qw, sc, xa, u)
    part = O.q_prefill_xasym(qw, sc, xa, u[:, :20])
    step = O.q_decode_xasym(qw, sc, xa, u[:, 20], part["h"], part["conv_state"])
    a, b = step["out"][:, 0].astype(np.float64), full["out"][:, 20].astype(np.float64)
    assert np.abs(a - b).max() <= 2e-2 * np.abs(b).max()
    assert np.abs(step["h"] - full["h"]).max() <= 2e-2 * np.abs(full["h"]).max()
    assert np.array_equal(step["conv_state"].view(np.uint16), full["conv_state"].view(np.uint16))
