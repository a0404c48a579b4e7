"""GPU parity of the asymmetric scan-input grid (Appendix K, "MinMax Asym. Per."): calibration, and
the prefill / decode chains link by link.  Bars as for the main path: x_proj with its column
correction and dt_proj bit for bit on the GPU's own codes, conv codes within 1 LSB on <= 0.1 %,
scan output <= 1e-3."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2410_13229_amd as Q
import workloads as W
from gpu_util import assert_lsb, dev, empty, host, make_taps, qweights_to_dev, rel_err, workspace

pytestmark = pytest.mark.gpu


def _setup(name):
    if name == "tiny":
        cfg = W.tiny_config(name="ta", d_model=64, d_inner=192, dt_rank=16, config_id=96)
    else:
        cfg = W.CONFIGS[name]
    w = W.make_weights(cfg, randomize_bias=True)
    calib = W.make_calibration(cfg)
    return cfg, w, calib, O.calibrate_xasym(w, calib)


@pytest.mark.parametrize("name", ["tiny", "c0"])
def test_calibrate_xasym_matches_oracle(name):
    cfg, w, calib, (qw_ref, sc_ref, xa_ref) = _setup(name)
    fw = {k: dev(v) for k, v in w.items()}
    out_q = {k: torch.zeros(v.shape, dtype=torch.int8 if v.dtype == np.int8 else torch.float32, device="cuda:0")
             for k, v in qw_ref.items()}
    col_bias = torch.zeros(xa_ref["col_bias"].shape, dtype=torch.int32, device="cuda:0")
    nb, Lc = calib.shape[:2]
    ws = workspace(Q.quamba_calibrate_workspace_bytes(cfg, nb, Lc))
    sc, xa = Q.quamba_calibrate_xasym(cfg, fw, dev(calib), nb, Lc, 99.999, out_q, col_bias, ws)
    got = Q.xasym_to_dict(xa)
    for k in Q.XASYM_FIELDS:
        assert abs(got[k] - float(xa_ref[k])) <= 2e-3 * abs(float(xa_ref[k])), (k, got[k], float(xa_ref[k]))
    assert abs(got["zero_point"] - xa_ref["zero_point"]) <= 1
    # the column term is exact for the GPU's own zero point and quantized weight
    wx = host(out_q["W_x"]).astype(np.int64)
    assert np.array_equal(host(col_bias).astype(np.int64), -got["zero_point"] * wx.sum(axis=1))


def _run(cfg, qw, sc, xa, u, decode_state=None, h0=None):
    decode = decode_state is not None
    Bt = u.shape[0]
    L = 1 if decode else u.shape[1]
    M = Bt * L
    qd = qweights_to_dev(qw)
    cb = dev(xa["col_bias"])
    xas = Q.make_xasym(cb, xa)
    taps = make_taps(cfg, M, ["xz_q", "x_q", "acc_x", "dbc_q", "dt_q", "y_f32", "g16", "gH_q"])
    ws = workspace(Q.quamba_workspace_bytes(cfg, Bt, L))
    out = empty((Bt, L, cfg.d_model), torch.float16)
    if decode:
        ssm, cs = dev(decode_state["ssm_state"]), dev(decode_state["conv_state"])
        Q.quamba_mixer_decode_xasym(cfg, qd, sc, xas, dev(u), Bt, out, ssm, cs, taps, ws)
    else:
        ssm = dev(h0) if h0 is not None else torch.zeros((Bt, cfg.d_inner, cfg.d_state), dtype=torch.float32, device="cuda:0")
        cs = empty((Bt, cfg.d_inner, cfg.d_conv - 1), torch.float16)
        Q.quamba_mixer_prefill_xasym(cfg, qd, sc, xas, dev(u), Bt, L, out, ssm, cs, taps, ws)
    r = {"out": host(out), "h": host(ssm), "conv_state": host(cs)}
    r.update({k: host(v) for k, v in taps.items()})
    return r


def _check_links(cfg, qw, sc, xa, r, Bt, L, h0=None, decode_state=None):
    Di, N, R = cfg.d_inner, cfg.d_state, cfg.dt_rank
    xz3 = r["xz_q"].reshape(Bt, L, 2 * Di)
    if decode_state is None:
        x32 = O.mixer.conv_prefill_silu(xz3[:, :, :Di], qw["conv_w"], qw["conv_b"], sc)
    else:
        x32, _ = O.mixer.conv_step_silu(xz3[:, 0, :Di], decode_state["conv_state"], qw["conv_w"], qw["conv_b"], sc)
    assert_lsb(r["x_q"], O.quantize_asym(x32, xa["inv_s_x"], xa["zero_point"]).reshape(Bt * L, Di), "x_q")
    acc = O.int_matmul(r["x_q"], qw["W_x"])
    assert np.array_equal(r["acc_x"], acc)  # the tap holds the raw sums
    accc = (acc.astype(np.int64) + xa["col_bias"].astype(np.int64)).astype(np.int32)
    assert np.array_equal(r["dbc_q"][:, :R], O.requant_acc(accc[:, :R], xa["m_x_dt"]))
    assert np.array_equal(r["dbc_q"][:, R:R + N], O.requant_acc(accc[:, R:R + N], xa["m_x_B"]))
    assert np.array_equal(r["dbc_q"][:, R + N:], O.requant_acc(accc[:, R + N:], xa["m_x_C"]))
    assert np.array_equal(r["dt_q"], O.requant_acc(O.int_matmul(r["dbc_q"][:, :R], qw["W_dt"]), sc["m_dt"]))
    dbc3 = r["dbc_q"].reshape(Bt, L, R + 2 * N)
    hh = decode_state["ssm_state"] if decode_state is not None else h0
    x_deq = np.float32(xa["s_x"]) * (r["x_q"].astype(np.float32) - np.float32(xa["zero_point"]))
    g_ref, _, h_ref = O.q_scan(None, r["dt_q"].reshape(Bt, L, Di), xz3[:, :, Di:], dbc3[..., R:R + N], dbc3[..., R + N:],
                               qw["A"], qw["D"], qw["dt_bias"], sc, hh, x_values=x_deq.reshape(Bt, L, Di))
    assert rel_err(r["y_f32"].reshape(Bt, L, Di), g_ref) <= 1e-3
    assert rel_err(r["h"], h_ref) <= 1e-3
    _, gHq_ref = O.q_hadamard_quant(r["g16"], sc)
    assert_lsb(r["gH_q"], gHq_ref, "gH_q")
    _, out = O.q_out_proj(r["gH_q"], qw["W_outH"], sc)
    assert np.array_equal(r["out"].reshape(Bt * L, -1).view(np.uint16), out.view(np.uint16))


@pytest.mark.parametrize("name,Bt,L", [("tiny", 3, 37), ("tiny", 1, 1), ("c0", 2, 130)])
def test_prefill_xasym_chain(name, Bt, L):
    cfg, w, calib, (qw, sc, xa) = _setup(name)
    u = W.make_hidden(cfg, batch=Bt, seqlen=L, stream=21)
    h0 = (np.random.default_rng(1).standard_normal((Bt, cfg.d_inner, cfg.d_state)) * 0.1).astype(np.float32)
    r = _run(cfg, qw, sc, xa, u, h0=h0)
    _check_links(cfg, qw, sc, xa, r, Bt, L, h0=h0)
    ref = O.q_prefill_xasym(qw, sc, xa, u, h0=h0)
    assert rel_err(r["out"].astype(np.float64), ref["out"].astype(np.float64)) <= 2e-2
    assert np.array_equal(r["conv_state"].view(np.uint16), ref["conv_state"].view(np.uint16))


@pytest.mark.parametrize("name,Bt", [("tiny", 3), ("tiny", 9), ("c0", 64)])
def test_decode_xasym_chain(name, Bt):
    cfg, w, calib, (qw, sc, xa) = _setup(name)
    ssm0, cs0 = W.make_decode_state(cfg, batch=Bt)
    u = W.make_hidden(cfg, batch=Bt, seqlen=1, stream=33)[:, 0]
    st = {"ssm_state": ssm0, "conv_state": cs0}
    r = _run(cfg, qw, sc, xa, u, decode_state=st)
    _check_links(cfg, qw, sc, xa, r, Bt, 1, decode_state=st)
    ref = O.q_decode_xasym(qw, sc, xa, u, ssm0, cs0)
    assert rel_err(r["out"].astype(np.float64), ref["out"].astype(np.float64)) <= 2e-2


def test_zero_point_zero_is_the_symmetric_path():
    """With zero point 0, no column term and Quamba's own scale the entry point reproduces
    quamba_mixer_prefill bit for bit."""
    cfg, w, calib, (qw, sc, xa) = _setup("tiny")
    u = W.make_hidden(cfg, batch=2, seqlen=40, stream=3)
    sym = dict(xa, zero_point=0, s_x=sc["s_x"], inv_s_x=sc["inv_s_x"], m_x_dt=sc["m_x_dt"], m_x_B=sc["m_x_B"],
               m_x_C=sc["m_x_C"], col_bias=np.zeros_like(xa["col_bias"]))
    a = _run(cfg, qw, sc, sym, u)
    from gpu_util import run_prefill
    b = run_prefill(cfg, qweights_to_dev(qw), sc, u, taps=False)
    assert np.array_equal(a["out"].view(np.uint16), b["out"].view(np.uint16))
    assert np.array_equal(a["h"], b["h"])


def test_xasym_argument_errors():
    cfg, w, calib, (qw, sc, xa) = _setup("tiny")
    qd = qweights_to_dev(qw)
    xas = Q.make_xasym(dev(xa["col_bias"]), xa)
    xas.col_bias = None
    u = dev(W.make_hidden(cfg, batch=1, seqlen=8))
    out = empty((1, 8, cfg.d_model), torch.float16)
    with pytest.raises(Q.QuambaError):
        Q.quamba_mixer_prefill_xasym(cfg, qd, sc, xas, u, 1, 8, out, None, None, None,
                                     workspace(Q.quamba_workspace_bytes(cfg, 1, 8)))
