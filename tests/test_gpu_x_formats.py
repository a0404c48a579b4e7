"""GPU parity of the non-uniform 8-bit formats of the scan input (Appendix K: log2 and E4M3): the
encoders bit for bit (integer decisions on the bits of an fp32 value), x_proj on the bf16 matrix units
against the float64 product (fp32 sums: within 2e-5 of the largest sum; the int8 outputs exact on the
GPU's own sums and within 1 LSB on <= 0.1 % of the oracle's), calibration, and the prefill / decode
chains link by link with the bars of the main path."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2410_13229_amd as Q
import workloads as W
from gpu_util import assert_lsb, dev, empty, host, make_taps, qweights_to_dev, rel_err, workspace
from oracle import x_formats as XF

pytestmark = pytest.mark.gpu

FMT_ID = {"e4m3": Q.XFMT_E4M3, "log2": Q.XFMT_LOG2}


def _order_index(fmt, code):
    """Codes -> integers that order like the values they stand for (adjacent values differ by one)."""
    c = np.asarray(code).astype(np.int64)
    mag = (c & 0x7F) if fmt == "e4m3" else 127 - (c & 0x7F)
    return np.where(c & 0x80, -mag, mag)


def _bf16_bits(w_q):
    """int8 codes [N, K] -> bfloat16 bit patterns in the order the header documents:
    out[(s N + n) 16 + 8 h + j] = W[n, 32 (s // 2) + 16 h + 8 (s % 2) + j]."""
    w = np.asarray(w_q)
    N, K = w.shape
    bits = (w.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    s, h, j = np.meshgrid(np.arange(K // 16), np.arange(2), np.arange(8), indexing="ij")
    k = (32 * (s // 2) + 16 * h + 8 * (s % 2) + j).reshape(K // 16, 16)           # [s, 8 h + j] -> k
    return np.ascontiguousarray(bits[:, k].transpose(1, 0, 2)).reshape(N, K)      # [s, n, p], kept 2-D for the allocators


def _encode_on_gpu(fmt, v, inv_s):
    v = np.ascontiguousarray(v, dtype=np.float32)
    codes = torch.zeros(v.size, dtype=torch.uint8, device="cuda:0")
    Q.quamba_x_encode(FMT_ID[fmt], dev(v), v.size, inv_s, codes)
    return host(codes)


@pytest.mark.parametrize("fmt", XF.FORMATS)
def test_encoder_bit_exact(fmt):
    rng = np.random.default_rng(11)
    table = XF.decode_e4m3(np.arange(0x7F))
    mids = (table[1:] + table[:-1]) / 2
    pows = np.exp2(-np.arange(0, 150, dtype=np.float64))
    r2 = float(np.float32(1.4142135623730951))
    pieces = [table, mids, mids * (1 - 2.0 ** -20), mids * (1 + 2.0 ** -20), pows, pows * r2,
              np.nextafter(np.float32(pows[:120] * r2), np.float32(0)).astype(np.float64),
              np.nextafter(np.float32(pows[:120] * r2), np.float32(4)).astype(np.float64),
              rng.standard_normal(20000) * 3, rng.standard_normal(5000) * 300, rng.standard_normal(5000) * 1e-3,
              np.exp2(rng.uniform(-149, 9, 20000)), [0.0, 448.0, 449.0, 463.9, 464.0, 465.0, 1e30, 1e-44, 2.0 ** -126.4]]
    v = np.concatenate([np.asarray(p, dtype=np.float64) for p in pieces])
    v = np.concatenate([v, -v]).astype(np.float32)
    assert np.array_equal(_encode_on_gpu(fmt, v, 1.0), XF.encode(fmt, v, 1.0))
    for inv_s in (0.37, 123.456, 1.0 / 448.0):
        w = (rng.standard_normal(30000) * 2).astype(np.float32)
        assert np.array_equal(_encode_on_gpu(fmt, w, inv_s), XF.encode(fmt, w, inv_s))


@pytest.mark.parametrize("fmt", XF.FORMATS)
@pytest.mark.parametrize("M,N,K", [(1, 48, 64), (37, 80, 192), (64, 192, 5120), (200, 192, 5120), (2048, 192, 5120),
                                   (4100, 192, 1024), (70, 288, 1024), (5, 320, 32), (33, 192, 352)])
def test_xfmt_proj_against_the_float64_product(fmt, M, N, K):
    rng = np.random.default_rng(M + N + K)
    t = (rng.standard_normal((M, K)) * np.exp(rng.standard_normal((M, K)))).astype(np.float32)
    codes = XF.encode(fmt, t, 0.25)
    Wq = rng.integers(-128, 128, size=(N, K)).astype(np.int8)
    e0, e1 = (N // 8) * 4, (N // 8) * 4 + 16
    ref = XF.x_proj_real(codes, Wq, fmt)
    scale = 100.0 / np.abs(ref).max()
    mult = [scale, scale * 0.5, scale * 2.0]
    out = torch.zeros((M, N), dtype=torch.int8, device="cuda:0")
    acc = torch.zeros((M, N), dtype=torch.float32, device="cuda:0")
    for ws in (workspace(Q.quamba_gemm_workspace_bytes(M, N, K)), None):    # with and without the K split
        out.zero_()
        acc.zero_()
        Q.quamba_xfmt_proj(FMT_ID[fmt], dev(codes), M, N, K, dev(_bf16_bits(Wq)), e0, e1, mult, out, acc, ws)
        a = host(acc)
        assert rel_err(a, ref) <= 2e-5
        m = np.where(np.arange(N) < e0, mult[0], np.where(np.arange(N) < e1, mult[1], mult[2])).astype(np.float32)
        own = np.clip(np.rint(a * m[None, :]), -128, 127).astype(np.int8)
        assert np.array_equal(host(out), own)
        want = np.clip(np.rint(ref.astype(np.float32) * m[None, :]), -128, 127).astype(np.int8)
        assert_lsb(host(out), want, "x_proj codes")


def test_xfmt_proj_rejects_bad_arguments():
    codes = torch.zeros((4, 64), dtype=torch.uint8, device="cuda:0")
    Wb = torch.zeros((8, 64), dtype=torch.int16, device="cuda:0")
    out = torch.zeros((4, 8), dtype=torch.int8, device="cuda:0")
    for kw in (dict(fmt=7), dict(N=6), dict(K=48), dict(N=324)):
        a = dict(fmt=Q.XFMT_LOG2, N=8, K=64)
        a.update(kw)
        with pytest.raises(Q.QuambaError):
            Q.quamba_xfmt_proj(a["fmt"], codes, 4, a["N"], a["K"], Wb, 4, 8, [1.0, 1.0, 1.0], out, None, None)


def _setup(name, fmt):
    cfg = W.tiny_config(name="tf", d_model=64, d_inner=192, dt_rank=16, config_id=95) if name == "tiny" else W.CONFIGS[name]
    w = W.make_weights(cfg, randomize_bias=True)
    calib = W.make_calibration(cfg)
    return cfg, w, calib, XF.calibrate_xfmt(w, calib, fmt)


@pytest.mark.parametrize("fmt", XF.FORMATS)
@pytest.mark.parametrize("name", ["tiny", "c0"])
def test_calibrate_xfmt_matches_oracle(name, fmt):
    cfg, w, calib, (qw_ref, sc_ref, xf_ref) = _setup(name, fmt)
    fw = {k: dev(v) for k, v in w.items()}
    out_q = {k: torch.zeros(v.shape, dtype=torch.int8 if v.dtype == np.int8 else torch.float32, device="cuda:0")
             for k, v in qw_ref.items()}
    wb = torch.zeros(qw_ref["W_x"].shape, dtype=torch.int16, device="cuda:0")
    nb, Lc = calib.shape[:2]
    ws = workspace(Q.quamba_calibrate_workspace_bytes(cfg, nb, Lc))
    sc, xf = Q.quamba_calibrate_xfmt(cfg, fw, dev(calib), nb, Lc, FMT_ID[fmt], 99.999, out_q, wb, ws)
    got = Q.xfmt_to_dict(xf)
    assert got["format"] == FMT_ID[fmt]
    for k in Q.XFMT_FIELDS:
        assert abs(got[k] - float(xf_ref[k])) <= 2e-3 * abs(float(xf_ref[k])), (k, got[k], float(xf_ref[k]))
    assert np.array_equal(host(wb).view(np.uint16), _bf16_bits(host(out_q["W_x"])))


def _run(cfg, qw, sc, xf, u, decode_state=None, h0=None):
    decode = decode_state is not None
    Bt = u.shape[0]
    L = 1 if decode else u.shape[1]
    M = Bt * L
    qd = qweights_to_dev(qw)
    wb = dev(_bf16_bits(qw["W_x"]).view(np.int16))
    xfs = Q.make_xfmt(wb, dict(xf, format=FMT_ID[xf["fmt"]]))
    taps = make_taps(cfg, M, ["xz_q", "x_q", "acc_x", "dbc_q", "dt_q", "y_f32", "g16", "gH_q"])
    ws = workspace(Q.quamba_workspace_bytes(cfg, Bt, L))
    out = empty((Bt, L, cfg.d_model), torch.float16)
    if decode:
        ssm, cs = dev(decode_state["ssm_state"]), dev(decode_state["conv_state"])
        Q.quamba_mixer_decode_xfmt(cfg, qd, sc, xfs, dev(u), Bt, out, ssm, cs, taps, ws)
    else:
        ssm = dev(h0) if h0 is not None else torch.zeros((Bt, cfg.d_inner, cfg.d_state), dtype=torch.float32, device="cuda:0")
        cs = empty((Bt, cfg.d_inner, cfg.d_conv - 1), torch.float16)
        Q.quamba_mixer_prefill_xfmt(cfg, qd, sc, xfs, dev(u), Bt, L, out, ssm, cs, taps, ws)
    r = {"out": host(out), "h": host(ssm), "conv_state": host(cs)}
    r.update({k: host(v) for k, v in taps.items()})
    return r


def _check_links(cfg, qw, sc, xf, r, Bt, L, h0=None, decode_state=None):
    Di, N, R = cfg.d_inner, cfg.d_state, cfg.dt_rank
    fmt = xf["fmt"]
    xz3 = r["xz_q"].reshape(Bt, L, 2 * Di)
    if decode_state is None:
        x32 = O.mixer.conv_prefill_silu(xz3[:, :, :Di], qw["conv_w"], qw["conv_b"], sc)
    else:
        x32, _ = O.mixer.conv_step_silu(xz3[:, 0, :Di], decode_state["conv_state"], qw["conv_w"], qw["conv_b"], sc)
    codes = r["x_q"].view(np.uint8)
    assert not np.any((codes & 0x7F) == 0x7F) or fmt == "log2"              # E4M3: never a not-a-number code
    assert_lsb(_order_index(fmt, codes), _order_index(fmt, XF.encode(fmt, x32, xf["inv_s_x"]).reshape(Bt * L, Di)), "x codes")
    acc = r["acc_x"].view(np.float32)                                       # the tap holds the fp32 sums
    assert rel_err(acc, XF.x_proj_real(codes, qw["W_x"], fmt)) <= 2e-5
    assert np.array_equal(r["dbc_q"][:, :R], XF.requant_real(acc[:, :R], xf["m_x_dt"]))
    assert np.array_equal(r["dbc_q"][:, R:R + N], XF.requant_real(acc[:, R:R + N], xf["m_x_B"]))
    assert np.array_equal(r["dbc_q"][:, R + N:], XF.requant_real(acc[:, R + N:], xf["m_x_C"]))
    assert np.array_equal(r["dt_q"], O.requant_acc(O.int_matmul(r["dbc_q"][:, :R], qw["W_dt"]), sc["m_dt"]))
    dbc3 = r["dbc_q"].reshape(Bt, L, R + 2 * N)
    hh = decode_state["ssm_state"] if decode_state is not None else h0
    x_deq = (np.float32(xf["s_x"]) * XF.decode(fmt, codes).astype(np.float32)).astype(np.float32)
    g_ref, _, h_ref = O.q_scan(None, r["dt_q"].reshape(Bt, L, Di), xz3[:, :, Di:], dbc3[..., R:R + N], dbc3[..., R + N:],
                               qw["A"], qw["D"], qw["dt_bias"], sc, hh, x_values=x_deq.reshape(Bt, L, Di))
    assert rel_err(r["y_f32"].reshape(Bt, L, Di), g_ref) <= 1e-3
    assert rel_err(r["h"], h_ref) <= 1e-3
    _, gHq_ref = O.q_hadamard_quant(r["g16"], sc)
    assert_lsb(r["gH_q"], gHq_ref, "gH_q")
    _, out = O.q_out_proj(r["gH_q"], qw["W_outH"], sc)
    assert np.array_equal(r["out"].reshape(Bt * L, -1).view(np.uint16), out.view(np.uint16))


@pytest.mark.parametrize("fmt", XF.FORMATS)
@pytest.mark.parametrize("name,Bt,L", [("tiny", 3, 37), ("tiny", 1, 1), ("c0", 2, 130)])
def test_prefill_xfmt_chain(name, Bt, L, fmt):
    cfg, w, calib, (qw, sc, xf) = _setup(name, fmt)
    u = W.make_hidden(cfg, batch=Bt, seqlen=L, stream=21)
    h0 = (np.random.default_rng(1).standard_normal((Bt, cfg.d_inner, cfg.d_state)) * 0.1).astype(np.float32)
    r = _run(cfg, qw, sc, xf, u, h0=h0)
    _check_links(cfg, qw, sc, xf, r, Bt, L, h0=h0)
    ref = XF.q_prefill_xfmt(qw, sc, xf, u, h0=h0)
    assert rel_err(r["out"].astype(np.float64), ref["out"].astype(np.float64)) <= 2e-2
    assert np.array_equal(r["conv_state"].view(np.uint16), ref["conv_state"].view(np.uint16))


@pytest.mark.parametrize("fmt", XF.FORMATS)
@pytest.mark.parametrize("name,Bt", [("tiny", 3), ("tiny", 19), ("c0", 64)])
def test_decode_xfmt_chain(name, Bt, fmt):
    cfg, w, calib, (qw, sc, xf) = _setup(name, fmt)
    ssm0, cs0 = W.make_decode_state(cfg, batch=Bt)
    u = W.make_hidden(cfg, batch=Bt, seqlen=1, stream=33)[:, 0]
    st = {"ssm_state": ssm0, "conv_state": cs0}
    r = _run(cfg, qw, sc, xf, u, decode_state=st)
    _check_links(cfg, qw, sc, xf, r, Bt, 1, decode_state=st)
    ref = XF.q_decode_xfmt(qw, sc, xf, u, ssm0, cs0)
    assert rel_err(r["out"].astype(np.float64), ref["out"].astype(np.float64)) <= 2e-2


@pytest.mark.parametrize("fmt", XF.FORMATS)
def test_prefill_xfmt_2p8b_width_sampled(fmt):
    """The width and token count the benchmark times (c1), checked link by link."""
    cfg = W.CONFIGS["c1"]
    w = W.make_weights(cfg, randomize_bias=True)
    qw, sc, xf = XF.calibrate_xfmt(w, W.make_calibration(cfg), fmt)
    u = W.make_hidden(cfg, batch=1, seqlen=256, stream=5)
    r = _run(cfg, qw, sc, xf, u)
    _check_links(cfg, qw, sc, xf, r, 1, 256)


def test_xfmt_argument_errors():
    cfg, w, calib, (qw, sc, xf) = _setup("tiny", "log2")
    qd = qweights_to_dev(qw)
    wb = dev(_bf16_bits(qw["W_x"]).view(np.int16))
    u = dev(W.make_hidden(cfg, batch=1, seqlen=8))
    out = empty((1, 8, cfg.d_model), torch.float16)
    ws = workspace(Q.quamba_workspace_bytes(cfg, 1, 8))
    bad = Q.make_xfmt(wb, dict(xf, format=9))
    with pytest.raises(Q.QuambaError):
        Q.quamba_mixer_prefill_xfmt(cfg, qd, sc, bad, u, 1, 8, out, None, None, None, ws)
    null = Q.make_xfmt(wb, dict(xf, format=Q.XFMT_LOG2))
    null.W_x_bf16 = None
    with pytest.raises(Q.QuambaError):
        Q.quamba_mixer_prefill_xfmt(cfg, qd, sc, null, u, 1, 8, out, None, None, None, ws)
