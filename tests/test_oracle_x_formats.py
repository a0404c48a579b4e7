"""Pins for the oracle's non-uniform 8-bit formats of the scan input (Appendix K: "MinMax Sym. Log2"
and the E4M3 float the appendix names as an alternative)."""
import dataclasses
from fractions import Fraction

import numpy as np
import pytest

import oracle as O
import workloads as W
from oracle import x_formats as XF


def _setup(outlier_gain=None, **kw):
    cfg = W.tiny_config(name="tf", d_model=64, d_inner=192, dt_rank=16, config_id=95, **kw)
    if outlier_gain is not None:
        cfg = dataclasses.replace(cfg, outlier_gain=outlier_gain)
    w = W.make_weights(cfg, randomize_bias=True)
    return cfg, w, W.make_calibration(cfg)


# ------------------------------------------------------------------------------------ E4M3
def test_e4m3_table_has_the_defining_numbers_of_the_format():
    """1-4-3 bits, bias 7: 448 the largest finite value, 2^-6 the smallest normal, 2^-9 the smallest
    subnormal, 1.0 at 0x38, eight mantissa steps per binade, two not-a-number codes and no infinity."""
    v = XF.decode_e4m3(np.arange(256))
    assert np.isnan(v[0x7F]) and np.isnan(v[0xFF]) and np.count_nonzero(np.isnan(v)) == 2
    assert not np.any(np.isinf(v))
    pos = v[:0x7F]
    assert pos[0] == 0.0 and pos[1] == 2.0 ** -9 and pos[7] == 7 * 2.0 ** -9 and pos[8] == 2.0 ** -6
    assert pos[0x38] == 1.0 and pos[0x39] == 1.125 and pos[0x40] == 2.0 and pos[0x7E] == 448.0
    assert np.all(np.diff(pos) > 0)                                   # codes order like their values
    assert np.array_equal(v[0x80:0xFF], -pos) and np.signbit(v[0x80])
    # spacing: 2^(E-3) inside the binade of 2^E
    for code in range(8, 0x7E):
        E = (code >> 3) - 7
        assert pos[code + 1] - pos[code] == 2.0 ** (E - 3)


def _nearest_in_table(t):
    """Brute force: the finite value closest to t; of two equally close ones the one with the even code."""
    table = XF.decode_e4m3(np.arange(0x7F))
    a = min(abs(float(t)), 448.0)
    d = np.abs(table - a)
    best = np.flatnonzero(d == d.min())
    code = int(best[0]) if len(best) == 1 else int([c for c in best if c % 2 == 0][0])
    return code | (0x80 if np.signbit(np.float32(t)) else 0)


def test_e4m3_encoder_is_the_nearest_value_with_ties_to_even():
    rng = np.random.default_rng(1)
    table = XF.decode_e4m3(np.arange(0x7F))
    mids = (table[1:] + table[:-1]) / 2                               # every tie of the format, exact in fp32
    near = np.concatenate([mids * (1 - 2.0 ** -20), mids * (1 + 2.0 ** -20)])
    samples = np.concatenate([table, mids, near, rng.standard_normal(4000) * 3, rng.standard_normal(2000) * 200,
                              rng.standard_normal(2000) * 0.01, [448.0, 449.0, 463.9, 464.0, 465.0, 1e9, 1e-12, 0.0]])
    samples = np.concatenate([samples, -samples]).astype(np.float32)
    got = XF.encode_e4m3(samples)
    want = np.array([_nearest_in_table(t) for t in samples], dtype=np.uint8)
    assert np.array_equal(got, want)
    assert not np.any((got & 0x7F) == 0x7F)                           # never a not-a-number code


def test_e4m3_round_trip_and_error_bounds():
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    vals = XF.decode_e4m3(codes)
    assert np.array_equal(XF.encode_e4m3(vals.astype(np.float32)), codes)
    rng = np.random.default_rng(2)
    t = np.exp(rng.uniform(np.log(2.0 ** -6), np.log(448.0), 20000)).astype(np.float32)
    back = XF.decode_e4m3(XF.encode_e4m3(t))
    assert np.max(np.abs(back - t) / t) <= 2.0 ** -4                  # half a mantissa step of 2^-3
    small = rng.uniform(0, 2.0 ** -6, 5000).astype(np.float32)
    assert np.max(np.abs(XF.decode_e4m3(XF.encode_e4m3(small)) - small)) <= 2.0 ** -10
    assert XF.decode_e4m3(XF.encode_e4m3(np.float32([1e6, -1e6]))).tolist() == [448.0, -448.0]


# ------------------------------------------------------------------------------------ log2
def test_log2_codes_powers_of_two_exactly_and_rounds_in_the_log_domain():
    e = np.arange(0, 127)
    p = np.exp2(-e.astype(np.float64)).astype(np.float32)
    assert np.array_equal(XF.encode_log2(p), e.astype(np.uint8))
    assert np.array_equal(XF.encode_log2(-p), (e | 0x80).astype(np.uint8))
    assert np.array_equal(XF.decode_log2(XF.encode_log2(p)), p.astype(np.float64))
    # brute force in the log domain: the exponent k minimising |log2 t - k|
    rng = np.random.default_rng(3)
    t = np.exp2(rng.uniform(-30, 0, 20000)).astype(np.float32)
    lg = np.log2(t.astype(np.float64))
    clear = np.abs(lg - np.floor(lg) - 0.5) > 1e-6                    # away from the tie, where fp32 sqrt 2 decides
    want = np.clip(-np.rint(lg), 0, 126).astype(np.uint8)
    assert np.array_equal(XF.encode_log2(t)[clear], want[clear])
    # the tie itself: fp32(sqrt 2) and its neighbours
    r2 = np.float32(1.4142135623730951)
    below, above = np.nextafter(r2, np.float32(0)), np.nextafter(r2, np.float32(2))
    assert XF.encode_log2(np.float32([below / 4, r2 / 4, above / 4])).tolist() == [2, 1, 1]


def test_log2_error_bound_saturation_and_zero():
    rng = np.random.default_rng(4)
    t = np.exp2(rng.uniform(-126, 0, 20000)).astype(np.float32)
    ratio = XF.decode_log2(XF.encode_log2(t)) / t.astype(np.float64)
    assert ratio.max() <= 2 ** 0.5 * (1 + 1e-6) and ratio.min() >= 2 ** -0.5 * (1 - 1e-6)
    assert XF.encode_log2(np.float32([1.0, 1.3, 1.5, 7.0, 1e20])).tolist() == [0, 0, 0, 0, 0]      # beyond the scale
    z = XF.encode_log2(np.float32([0.0, -0.0, 1e-45, -(2.0 ** -127.5)]))
    assert z.tolist() == [127, 127, 127, 127] and np.all(XF.decode_log2(z) == 0)
    assert XF.encode_log2(np.float32([2.0 ** -126, 2.0 ** -126.4])).tolist() == [126, 126]


# ------------------------------------------------------------------------------------ x_proj
@pytest.mark.parametrize("fmt", XF.FORMATS)
def test_x_proj_on_decoded_values_is_the_exact_rational_dot_product(fmt):
    rng = np.random.default_rng(5)
    codes = rng.integers(0, 256, size=(4, 40)).astype(np.uint8)
    codes[(codes & 0x7F) == 0x7F] = 0x10
    if fmt == "log2":
        codes = (codes & 0x80) | (codes & 0x1F)                      # exponents up to 31: exact in float64 sums
    Wq = rng.integers(-128, 128, size=(6, 40)).astype(np.int8)
    got = XF.x_proj_real(codes, Wq, fmt)
    vals = XF.decode(fmt, codes)
    for m in range(4):
        for n in range(6):
            exact = sum(Fraction(int(Wq[n, k])) * Fraction(float(vals[m, k])) for k in range(40))
            assert Fraction(float(got[m, n])) == exact


def test_decoded_values_and_weight_codes_fit_bfloat16():
    """The device feeds both operands of x_proj to a bf16 matrix unit: eight significant bits hold
    every E4M3 value, every power of two down to 2^-126 and every int8 code exactly."""
    def bf16_round_trip(v):
        b = np.asarray(v, dtype=np.float32).view(np.uint32)
        return (b & np.uint32(0xFFFF0000)).view(np.float32), (b & np.uint32(0xFFFF)) == 0
    for vals in (XF.decode_e4m3(np.array([c for c in range(256) if (c & 0x7F) != 0x7F])),
                 XF.decode_log2(np.arange(256)), np.arange(-128, 128).astype(np.float64)):
        back, exact = bf16_round_trip(vals)
        assert np.all(exact) and np.array_equal(back.astype(np.float64), vals)


# ------------------------------------------------------------------------------------ mixer
@pytest.mark.parametrize("fmt", XF.FORMATS)
def test_calibrated_scale_follows_the_format(fmt):
    cfg, w, calib = _setup()
    qw, sc, xf = XF.calibrate_xfmt(w, calib, fmt)
    x = O.fp_forward(w, calib)["x"]
    if fmt == "e4m3":
        assert float(xf["s_x"]) == pytest.approx(O.percentile_max(x, 99.999) / 448.0, rel=1e-6)
    else:
        assert float(xf["s_x"]) == pytest.approx(np.abs(x).max(), rel=1e-6)
    # same weights and other scales as Quamba
    qw0, sc0 = O.calibrate(w, calib)
    assert all(np.array_equal(qw[k], qw0[k]) for k in qw0) and sc == sc0


@pytest.mark.parametrize("fmt", XF.FORMATS)
def test_variant_tracks_the_unquantized_mixer_and_decode_continues_prefill(fmt):
    cfg, w, calib = _setup()
    qw, sc, xf = XF.calibrate_xfmt(w, calib, fmt)
    u = W.make_hidden(cfg, batch=2, seqlen=40, stream=7)
    ref = O.fp_forward(w, u)
    full = XF.q_prefill_xfmt(qw, sc, xf, u)
    rel = np.linalg.norm(full["out"].astype(np.float64) - ref["out"]) / np.linalg.norm(ref["out"])
    base = O.q_prefill(qw, sc, u)
    rel0 = np.linalg.norm(base["out"].astype(np.float64) - ref["out"]) / np.linalg.norm(ref["out"])
    # E4M3 keeps three mantissa bits (2^-4 relative) and stays on par with the int8 grid; log2 keeps
    # none: a relative error uniform in the log domain, 0.2 rms on every x, bounds what it can reach
    # on well-behaved inputs (its case is heavy tails, pinned below)
    assert rel <= (max(2.0 * rel0, 0.1) if fmt == "e4m3" else 0.3)
    # a prefill of 39 tokens followed by one decode step is the 40-token prefill
    part = XF.q_prefill_xfmt(qw, sc, xf, u[:, :39])
    step = XF.q_decode_xfmt(qw, sc, xf, u[:, 39], part["h"], part["conv_state"])
    # (the step's conv reads an fp16 window, the prefill's the integer codes: the two x differ in the
    # last fp32 bits, which a few codes notice)
    assert np.mean(step["x_code"][:, 0] != full["x_code"][:, 39]) <= 0.02
    a, b = step["out"][:, 0].astype(np.float64), full["out"][:, 39].astype(np.float64)
    assert np.abs(a - b).max() <= 2e-2 * np.abs(b).max()
    assert np.abs(step["h"] - full["h"]).max() <= 2e-2 * np.abs(full["h"]).max()
    assert np.array_equal(step["conv_state"].view(np.uint16), full["conv_state"].view(np.uint16))


def test_x_reconstruction_error_by_format_on_outlier_inputs():
    """What Appendix K is about: x has a few large values.  The uniform absmax grid wastes its levels
    on them; the two non-uniform formats keep a relative accuracy for the small values whatever the
    largest one is (bounded relative error instead of bounded absolute error)."""
    cfg, w, calib = _setup(outlier_gain=100.0)
    x = O.fp_forward(w, calib)["x"].astype(np.float32)
    small = np.abs(x) < np.percentile(np.abs(x), 90)
    errs = {}
    for fmt in XF.FORMATS:
        qw, sc, xf = XF.calibrate_xfmt(w, calib, fmt)
        xh = float(xf["s_x"]) * XF.decode(fmt, XF.encode(fmt, x, xf["inv_s_x"]))
        errs[fmt] = np.linalg.norm((xh - x)[small]) / np.linalg.norm(x[small])
    s_abs = np.abs(x).max() / 127.0
    xq = np.clip(np.rint(x / s_abs), -128, 127) * s_abs
    errs["absmax"] = np.linalg.norm((xq - x)[small]) / np.linalg.norm(x[small])
    assert errs["e4m3"] <= 2.0 ** -4 * 1.05 or errs["e4m3"] < errs["absmax"]
    assert errs["log2"] <= (2 ** 0.5 - 1) * 1.05
    assert errs["e4m3"] < errs["log2"]                                # three mantissa bits against none
