"""Pins for the oracle's dynamic scan-input quantizer (Appendix K, "Dynamic / MinMax Sym.")."""
import dataclasses

import numpy as np

import oracle as O
import workloads as W
from oracle import x_dynamic as XD


def _setup(**kw):
    cfg = W.tiny_config(name="td", d_model=64, d_inner=192, dt_rank=16, config_id=94, **kw)
    w = W.make_weights(cfg, randomize_bias=True)
    return cfg, w, W.make_calibration(cfg)


def test_scale_is_eq2_on_the_calls_own_values():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal((3, 17, 64)) * 0.7).astype(np.float16)
    s, inv = XD.dynamic_scale(x)
    assert float(s) == float(np.float32(np.float32(np.abs(x.astype(np.float32)).max()) / np.float32(127)))
    assert float(inv) == float(np.float32(np.float32(1.0) / s))
    q = O.quantize(x.astype(np.float32), inv)
    i = np.unravel_index(np.argmax(np.abs(x.astype(np.float32))), x.shape)
    assert abs(int(q[i])) == 127 and np.abs(q.astype(np.int32)).max() == 127      # the largest value lands on the last code
    assert np.abs(float(s) * q.astype(np.float64) - x.astype(np.float64)).max() <= float(s) / 2 * 1.001
    # all-zero call: the paper does not cover it; the scale is 1 and every code 0
    s0, inv0 = XD.dynamic_scale(np.zeros((2, 2), np.float16))
    assert float(s0) == 1.0 and float(inv0) == 1.0


def test_codes_do_not_change_when_the_call_is_scaled_by_a_power_of_two():
    """The scale follows the data: x and 4 x get the same codes (a power of two commutes with every
    fp32 rounding above), which no static scale can do."""
    rng = np.random.default_rng(1)
    x = (rng.standard_normal((2, 9, 64)) * 0.3).astype(np.float16)
    s1, i1 = XD.dynamic_scale(x)
    s4, i4 = XD.dynamic_scale((x.astype(np.float32) * 4).astype(np.float16))
    assert float(s4) == 4 * float(s1)
    assert np.array_equal(O.quantize(x.astype(np.float32), i1), O.quantize(x.astype(np.float32) * 4, i4))


def test_dynamic_error_never_above_a_static_scale_from_other_data():
    rng = np.random.default_rng(2)
    calib = rng.standard_normal(4000) * 1.0
    for gain in (0.05, 0.3, 1.0):                       # the call's range is at most the calibration's
        x = (rng.standard_normal(4000) * gain).astype(np.float16)
        s, inv = XD.dynamic_scale(x)
        e_dyn = np.abs(float(s) * O.quantize(x.astype(np.float32), inv).astype(np.float64) - x.astype(np.float64)).max()
        ss = np.float32(np.abs(calib).max() / 127)
        e_sta = np.abs(float(ss) * O.quantize(x.astype(np.float32), np.float32(1 / ss)).astype(np.float64) - x.astype(np.float64)).max()
        assert e_dyn <= e_sta * 1.001
    assert float(XD.dynamic_scale((rng.standard_normal(100) * 0.05).astype(np.float16))[0]) < float(ss) / 5


def test_multipliers_follow_the_scale():
    cfg, w, calib = _setup()
    qw, sc = O.calibrate(w, calib)
    s = np.float32(0.0123)
    m = XD.dynamic_multipliers(s, sc)
    for got, k in zip(m, ("s_dtl", "s_B", "s_C")):
        assert abs(float(got) - float(s) * float(sc["s_Wx"]) / float(sc[k])) <= 1e-6 * abs(float(got))
    # with the calibrated scale itself they are Quamba's multipliers
    m0 = XD.dynamic_multipliers(sc["s_x"], sc)
    for got, k in zip(m0, ("m_x_dt", "m_x_B", "m_x_C")):
        assert abs(float(got) - float(sc[k])) <= 1e-6 * abs(float(sc[k]))


def test_tracks_the_unquantized_mixer_when_the_range_moves_and_decode_continues_prefill():
    """Calibrated on the usual inputs, evaluated on inputs 8 times smaller: the static scale of x
    (absmax rule) leaves most codes unused, the dynamic one adapts."""
    cfg, w, calib = _setup()
    qw, sc = O.calibrate(w, calib, x_percentile=100.0)
    u = (W.make_hidden(cfg, batch=2, seqlen=40, stream=7).astype(np.float32) / 8).astype(np.float16)
    ref = O.fp_forward(w, u)
    dyn = XD.q_prefill_xdyn(qw, sc, u)
    sta = O.q_prefill(qw, sc, u)
    x_ref = ref["x"]
    e_dyn = np.linalg.norm(dyn["x_deq"].astype(np.float64) - x_ref) / np.linalg.norm(x_ref)
    e_sta = np.linalg.norm(float(sc["s_x"]) * sta["x_q"].astype(np.float64) - x_ref) / np.linalg.norm(x_ref)
    assert e_dyn < e_sta
    part = XD.q_prefill_xdyn(qw, sc, u[:, :39])
    step = XD.q_decode_xdyn(qw, sc, u[:, 39], part["h"], part["conv_state"])
    full = XD.q_prefill_xdyn(qw, sc, u)
    assert np.array_equal(step["conv_state"].view(np.uint16), full["conv_state"].view(np.uint16))
    # (the step's scale is that of one token, the prefill's that of forty, and these inputs sit far below the
    # calibrated ranges of every other tensor: the two outputs agree to that quantization noise, and the
    # step is no further from the unquantized mixer than the prefill is)
    a, b = step["out"][:, 0].astype(np.float64), full["out"][:, 39].astype(np.float64)
    r = ref["out"][:, 39]
    assert np.abs(a - b).max() <= 0.25 * np.abs(b).max()
    assert np.abs(a - r).max() <= 1.5 * np.abs(b - r).max()
