"""GPU parity of the dynamic scan-input quantizer (Appendix K, "Dynamic / MinMax Sym."): the scale the
call derives from its own values bit for bit, the codes and multipliers formed from it bit for bit on the
GPU's own half-precision x, and the prefill / decode chains link by link with the bars of the main path."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2410_13229_amd as Q
import workloads as W
from gpu_util import assert_lsb, dev, empty, host, make_taps, qweights_to_dev, rel_err, workspace
from oracle import x_dynamic as XD

pytestmark = pytest.mark.gpu


def _setup(name):
    cfg = W.tiny_config(name="td", d_model=64, d_inner=192, dt_rank=16, config_id=94) if name == "tiny" else W.CONFIGS[name]
    w = W.make_weights(cfg, randomize_bias=True)
    return cfg, w, O.calibrate(w, W.make_calibration(cfg))


def _run(cfg, qw, sc, u, decode_state=None, h0=None):
    decode = decode_state is not None
    Bt = u.shape[0]
    L = 1 if decode else u.shape[1]
    M = Bt * L
    qd = qweights_to_dev(qw)
    taps = make_taps(cfg, M, ["xz_q", "x_q", "acc_x", "dbc_q", "dt_q", "y_f32", "g16", "gH_q"])
    ws = workspace(Q.quamba_xdyn_workspace_bytes(cfg, Bt, L))
    out = empty((Bt, L, cfg.d_model), torch.float16)
    s_out = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    x16 = empty((M, cfg.d_inner), torch.float16)
    if decode:
        ssm, cs = dev(decode_state["ssm_state"]), dev(decode_state["conv_state"])
        Q.quamba_mixer_decode_xdyn(cfg, qd, sc, dev(u), Bt, out, ssm, cs, taps, s_out, x16, ws)
    else:
        ssm = dev(h0) if h0 is not None else torch.zeros((Bt, cfg.d_inner, cfg.d_state), dtype=torch.float32, device="cuda:0")
        cs = empty((Bt, cfg.d_inner, cfg.d_conv - 1), torch.float16)
        Q.quamba_mixer_prefill_xdyn(cfg, qd, sc, dev(u), Bt, L, out, ssm, cs, taps, s_out, x16, ws)
    r = {"out": host(out), "h": host(ssm), "conv_state": host(cs), "s": host(s_out)[0], "x16": host(x16)}
    r.update({k: host(v) for k, v in taps.items()})
    return r


def _check_links(cfg, qw, sc, r, Bt, L, h0=None, decode_state=None):
    Di, N, R = cfg.d_inner, cfg.d_state, cfg.dt_rank
    xz3 = r["xz_q"].reshape(Bt, L, 2 * Di)
    if decode_state is None:
        x32 = O.mixer.conv_prefill_silu(xz3[:, :, :Di], qw["conv_w"], qw["conv_b"], sc)
    else:
        x32, _ = O.mixer.conv_step_silu(xz3[:, 0, :Di], decode_state["conv_state"], qw["conv_w"], qw["conv_b"], sc)
    # the conv output in half precision: the device's SiLU is a fast one, so a last-place difference is allowed
    want16 = x32.astype(np.float16).reshape(Bt * L, Di)
    d = np.abs(r["x16"].view(np.int16).astype(np.int32) - want16.view(np.int16).astype(np.int32))
    assert d.max() <= 1 and (d != 0).mean() <= 2e-3
    # from the GPU's own x16 on, everything is bit for bit: scale, codes, multipliers
    s, inv = XD.dynamic_scale(r["x16"])
    assert np.float32(r["s"]).view(np.uint32) == np.float32(s).view(np.uint32)
    assert np.array_equal(r["x_q"], O.quantize(r["x16"].astype(np.float32), inv))
    acc = O.int_matmul(r["x_q"], qw["W_x"])
    assert np.array_equal(r["acc_x"], acc)
    m_dt, m_B, m_C = XD.dynamic_multipliers(s, sc)
    assert np.array_equal(r["dbc_q"][:, :R], O.requant_acc(acc[:, :R], m_dt))
    assert np.array_equal(r["dbc_q"][:, R:R + N], O.requant_acc(acc[:, R:R + N], m_B))
    assert np.array_equal(r["dbc_q"][:, R + N:], O.requant_acc(acc[:, R + N:], m_C))
    assert np.array_equal(r["dt_q"], O.requant_acc(O.int_matmul(r["dbc_q"][:, :R], qw["W_dt"]), sc["m_dt"]))
    dbc3 = r["dbc_q"].reshape(Bt, L, R + 2 * N)
    hh = decode_state["ssm_state"] if decode_state is not None else h0
    x_deq = (np.float32(s) * r["x_q"].astype(np.float32)).astype(np.float32)
    g_ref, _, h_ref = O.q_scan(None, r["dt_q"].reshape(Bt, L, Di), xz3[:, :, Di:], dbc3[..., R:R + N], dbc3[..., R + N:],
                               qw["A"], qw["D"], qw["dt_bias"], sc, hh, x_values=x_deq.reshape(Bt, L, Di))
    assert rel_err(r["y_f32"].reshape(Bt, L, Di), g_ref) <= 1e-3
    assert rel_err(r["h"], h_ref) <= 1e-3
    _, gHq_ref = O.q_hadamard_quant(r["g16"], sc)
    assert_lsb(r["gH_q"], gHq_ref, "gH_q")
    _, out = O.q_out_proj(r["gH_q"], qw["W_outH"], sc)
    assert np.array_equal(r["out"].reshape(Bt * L, -1).view(np.uint16), out.view(np.uint16))


@pytest.mark.parametrize("name,Bt,L", [("tiny", 3, 37), ("tiny", 1, 1), ("c0", 2, 130), ("c1", 1, 256)])
def test_prefill_xdyn_chain(name, Bt, L):
    cfg, w, (qw, sc) = _setup(name)
    u = W.make_hidden(cfg, batch=Bt, seqlen=L, stream=21)
    h0 = (np.random.default_rng(1).standard_normal((Bt, cfg.d_inner, cfg.d_state)) * 0.1).astype(np.float32)
    r = _run(cfg, qw, sc, u, h0=h0)
    _check_links(cfg, qw, sc, r, Bt, L, h0=h0)
    ref = XD.q_prefill_xdyn(qw, sc, u, h0=h0)
    assert abs(float(r["s"]) - float(ref["s_x_dyn"])) <= 2e-3 * float(ref["s_x_dyn"])
    assert rel_err(r["out"].astype(np.float64), ref["out"].astype(np.float64)) <= 2e-2
    assert np.array_equal(r["conv_state"].view(np.uint16), ref["conv_state"].view(np.uint16))


@pytest.mark.parametrize("name,Bt", [("tiny", 3), ("tiny", 19), ("c0", 64), ("c2", 64)])
def test_decode_xdyn_chain(name, Bt):
    cfg, w, (qw, sc) = _setup(name)
    ssm0, cs0 = W.make_decode_state(cfg, batch=Bt)
    u = W.make_hidden(cfg, batch=Bt, seqlen=1, stream=33)[:, 0]
    st = {"ssm_state": ssm0, "conv_state": cs0}
    r = _run(cfg, qw, sc, u, decode_state=st)
    _check_links(cfg, qw, sc, r, Bt, 1, decode_state=st)
    ref = XD.q_decode_xdyn(qw, sc, u, ssm0, cs0)
    assert rel_err(r["out"].astype(np.float64), ref["out"].astype(np.float64)) <= 2e-2


def test_scale_follows_the_input_and_calls_do_not_leak_into_each_other():
    """A call on inputs 8 times smaller gets a clearly smaller scale (not 8 times: the conv bias and SiLU are
    not homogeneous), and running the large call again afterwards reproduces its first result bit for bit
    (the maximum is cleared per call)."""
    cfg, w, (qw, sc) = _setup("tiny")
    u = W.make_hidden(cfg, batch=2, seqlen=24, stream=4)
    small = (u.astype(np.float32) / 8).astype(np.float16)
    a = _run(cfg, qw, sc, u)
    b = _run(cfg, qw, sc, small)
    c = _run(cfg, qw, sc, u)
    assert float(b["s"]) < 0.7 * float(a["s"])
    assert np.array_equal(a["out"].view(np.uint16), c["out"].view(np.uint16)) and a["s"] == c["s"]


def test_xdyn_argument_errors():
    cfg, w, (qw, sc) = _setup("tiny")
    qd = qweights_to_dev(qw)
    u = dev(W.make_hidden(cfg, batch=1, seqlen=8))
    out = empty((1, 8, cfg.d_model), torch.float16)
    small = workspace(Q.quamba_workspace_bytes(cfg, 1, 8))      # the static path's workspace is too small
    assert Q.quamba_xdyn_workspace_bytes(cfg, 1, 8) > Q.quamba_workspace_bytes(cfg, 1, 8)
    with pytest.raises(Q.QuambaError):
        Q.quamba_mixer_prefill_xdyn(cfg, qd, sc, u, 1, 8, out, None, None, None, None, None, small)
