"""GPU parity of the whole quantized mixer through the C ABI (quamba_mixer_prefill /
quamba_mixer_decode / quamba_calibrate).

A single flipped int8 code upstream changes every accumulator downstream, so the chain is
checked link by link: every stage of the GPU run is compared with the oracle's stage function
applied to the GPU's own input to that stage (bit-exact for integer work, within the stated
tolerances for the floating-point stages), and the final fp16 output is also compared end to
end with the oracle's.  At the large shapes the same links are checked on sampled rows and
channels, which the oracle can compute one by one."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2410_13229_amd as Q
import workloads as W
from gpu_util import (assert_lsb, dev, empty, host, oracle_setup, qweights_to_dev, rel_err, run_prefill,
                      workspace, make_taps)

pytestmark = pytest.mark.gpu


def check_chain(cfg, qw, sc, u, r, h0=None, rows=None, chans=None, decode_state=None):
    """Verify each link of a GPU run `r` (taps as numpy, [M, cols]) against the oracle.
    rows: sampled token rows for the GEMM / Hadamard links (None = all);
    chans: sampled channels for the conv / scan links (None = all)."""
    Bt, L = u.shape[:2]
    Dm, Di, N, R = cfg.d_model, cfg.d_inner, cfg.d_state, cfg.dt_rank
    M = Bt * L
    rs = np.arange(M) if rows is None else np.asarray(rows)
    cs = np.arange(Di) if chans is None else np.asarray(chans)
    stats = {}
    # S0 quantize
    u_q = O.quantize(u.reshape(M, Dm)[rs].astype(np.float32), sc["inv_s_u"])
    assert np.array_equal(r["u_q"][rs], u_q)
    # S1 in_proj
    acc = O.int_matmul(r["u_q"][rs], qw["W_in"])
    if "acc_in" in r:  # the raw sums are absent when the run took the row-staged epilogues (as an untapped call does)
        assert np.array_equal(r["acc_in"][rs], acc)
    assert np.array_equal(r["xz_q"][rs, :Di], O.requant_acc(acc[:, :Di], sc["m_in_x"]))
    assert np.array_equal(r["xz_q"][rs, Di:], O.requant_acc(acc[:, Di:], sc["m_in_z"]))
    # S2 conv
    xz3 = r["xz_q"].reshape(Bt, L, 2 * Di)
    if decode_state is None:
        want = O.q_conv_prefill(xz3[:, :, cs], qw["conv_w"][cs], qw["conv_b"][cs], sc)
    else:
        want, _ = O.q_conv_step(xz3[:, 0, cs], decode_state["conv_state"][:, cs], qw["conv_w"][cs],
                                qw["conv_b"][cs], sc)
        want = want[:, None, :]
    got = r["x_q"].reshape(Bt, L, Di)[:, :, cs]
    assert_lsb(got, want, "x_q")
    stats["x_q_flip"] = float((got != want).mean())
    # S3 x_proj
    acc = O.int_matmul(r["x_q"][rs], qw["W_x"])
    if "acc_x" in r:
        assert np.array_equal(r["acc_x"][rs], acc)
    assert np.array_equal(r["dbc_q"][rs, :R], O.requant_acc(acc[:, :R], sc["m_x_dt"]))
    assert np.array_equal(r["dbc_q"][rs, R:R + N], O.requant_acc(acc[:, R:R + N], sc["m_x_B"]))
    assert np.array_equal(r["dbc_q"][rs, R + N:], O.requant_acc(acc[:, R + N:], sc["m_x_C"]))
    # S4 dt_proj
    acc = O.int_matmul(r["dbc_q"][rs, :R], qw["W_dt"])
    if "acc_dt" in r:  # absent when dt_proj ran inside the scan kernel (no raw sums to tap)
        assert np.array_equal(r["acc_dt"][rs], acc)
    assert np.array_equal(r["dt_q"][rs], O.requant_acc(acc, sc["m_dt"]))
    # S5 scan + gate
    dbc3 = r["dbc_q"].reshape(Bt, L, R + 2 * N)
    hh = decode_state["ssm_state"] if decode_state is not None else h0
    g_ref, g16_ref, h_ref = O.q_scan(r["x_q"].reshape(Bt, L, Di)[:, :, cs], r["dt_q"].reshape(Bt, L, Di)[:, :, cs],
                                     xz3[:, :, Di + cs], dbc3[..., R:R + N], dbc3[..., R + N:], qw["A"][cs],
                                     qw["D"][cs], qw["dt_bias"][cs], sc, None if hh is None else hh[:, cs])
    assert np.isfinite(g16_ref.astype(np.float32)).all(), "workload overflows fp16: not a valid parity case"
    if "y_f32" in r:
        stats["scan_err"] = rel_err(r["y_f32"].reshape(Bt, L, Di)[:, :, cs], g_ref)
        assert stats["scan_err"] <= 1e-3
    assert rel_err(r["g16"].reshape(Bt, L, Di)[:, :, cs].astype(np.float64), g_ref) <= 1e-3
    if "h" in r:
        assert rel_err(r["h"][:, cs], h_ref) <= 1e-3
    # S6 Hadamard + quant
    gH_ref, gHq_ref = O.q_hadamard_quant(r["g16"][rs], sc)
    if "gH_f32" in r:
        stats["had_err"] = rel_err(r["gH_f32"][rs], gH_ref)
        assert stats["had_err"] <= 1e-5
    assert_lsb(r["gH_q"][rs], gHq_ref, "gH_q")
    stats["gH_q_flip"] = float((r["gH_q"][rs] != gHq_ref).mean())
    # S7 out_proj
    acc, out = O.q_out_proj(r["gH_q"][rs], qw["W_outH"], sc)
    if "acc_out" in r:
        assert np.array_equal(r["acc_out"][rs], acc)
    assert np.array_equal(r["out"].reshape(M, Dm)[rs].view(np.uint16), out.view(np.uint16))
    return stats


def end_to_end(r, ref, name):
    """Final output against the oracle's own run.  The bound follows from the allowance of one
    code on 0.1 % of a requantized tensor: a flipped code moves a few downstream sums by one
    step of their scale, far below 2 % of the output's absmax."""
    e = rel_err(r["out"].astype(np.float64), ref["out"].astype(np.float64))
    assert e <= 2e-2, (name, e)
    return e


@pytest.mark.parametrize("Bt,L,dm,di,rk", [(2, 37, 64, 128, 16), (1, 5, 96, 192, 16), (3, 130, 160, 320, 32),
                                            (2, 1, 64, 128, 16),  # a prefill of one token
                                            # fewer channels than a workgroup, a ragged last chunk, the order-12 factor
                                            # with a wider dt_rank, five sequences
                                            (5, 257, 48, 32, 16), (1, 513, 128, 384, 48), (2, 64, 32, 640, 64)])
def test_prefill_tiny(Bt, L, dm, di, rk):
    cfg = W.tiny_config(name=f"t{di}", d_model=dm, d_inner=di, dt_rank=rk, batch=Bt, seqlen=L, config_id=91 + di)
    w, qw, sc = oracle_setup(cfg, randomize_bias=True, gain=4.0)
    u = W.make_hidden(cfg)
    rng = np.random.default_rng(5)
    h0 = (rng.standard_normal((Bt, di, 16)) * 0.1).astype(np.float32)
    r = run_prefill(cfg, qweights_to_dev(qw), sc, u, h0=h0)
    ref = O.q_prefill(qw, sc, u, h0=h0)
    check_chain(cfg, qw, sc, u, r, h0=h0)
    end_to_end(r, ref, cfg.name)
    assert np.array_equal(r["conv_state"].view(np.uint16), ref["conv_state"].view(np.uint16))
    assert rel_err(r["h"], ref["h"]) <= 2e-2
    # without the raw dt_proj sums among the taps the scan computes dt_q itself: same chain, same output
    from gpu_util import TAP_SHAPES
    r2 = run_prefill(cfg, qweights_to_dev(qw), sc, u, h0=h0, tap_names=[n for n in TAP_SHAPES if n != "acc_dt"])
    check_chain(cfg, qw, sc, u, r2, h0=h0)
    assert np.array_equal(r2["dt_q"], r["dt_q"])
    assert np.array_equal(r2["out"].view(np.uint16), r["out"].view(np.uint16))


def test_prefill_q_variant_and_null_state():
    cfg = W.tiny_config(name="tq", d_model=64, d_inner=128, dt_rank=16, batch=2, seqlen=20, config_id=95)
    w, qw, sc = oracle_setup(cfg, randomize_bias=True, gain=4.0)
    u = W.make_hidden(cfg)
    qd = qweights_to_dev(qw)
    a = run_prefill(cfg, qd, sc, u, want_state=False, taps=False)
    u_q = O.quantize(u.astype(np.float32), sc["inv_s_u"])
    b = run_prefill(cfg, qd, sc, None, u_q=u_q, want_state=True, taps=False)
    assert np.array_equal(a["out"].view(np.uint16), b["out"].view(np.uint16))


def test_prefill_c0_full():
    cfg = W.CONFIGS["c0"]
    w, qw, sc = oracle_setup(cfg)
    u = W.make_hidden(cfg)
    r = run_prefill(cfg, qweights_to_dev(qw), sc, u)
    ref = O.q_prefill(qw, sc, u)
    st = check_chain(cfg, qw, sc, u, r)
    e = end_to_end(r, ref, "c0")
    print("c0", st, "end-to-end", e)


def test_prefill_c1_full():
    cfg = W.CONFIGS["c1"]
    w, qw, sc = oracle_setup(cfg)
    u = W.make_hidden(cfg)
    r = run_prefill(cfg, qweights_to_dev(qw), sc, u)
    ref = O.q_prefill(qw, sc, u)
    st = check_chain(cfg, qw, sc, u, r)
    e = end_to_end(r, ref, "c1")
    print("c1", st, "end-to-end", e)


def _sampled(cfg, Bt, L, seed):
    rng = np.random.default_rng(seed)
    M = Bt * L
    rows = np.unique(np.concatenate([[0, 1, M - 1, M // 2], rng.integers(0, M, 60)]))
    chans = np.unique(np.concatenate([[0, 1, cfg.d_inner - 1], rng.integers(0, cfg.d_inner, 93)]))
    return rows, chans


def test_prefill_c4_full_size_sampled():
    """Jamba-shaped layer at L = 16384 in the launch configuration the benchmark uses."""
    cfg = W.CONFIGS["c4"]
    w, qw, sc = oracle_setup(cfg)
    u = W.make_hidden(cfg)
    r = run_prefill(cfg, qweights_to_dev(qw), sc, u)
    rows, chans = _sampled(cfg, cfg.batch, cfg.seqlen, 4)
    st = check_chain(cfg, qw, sc, u, r, rows=rows, chans=chans)
    print("c4", st)


def test_prefill_c3_layer_shape_sampled():
    """One layer of the 64-layer stack at its batch 4 x 4096 shape, with a carried-in state."""
    cfg = W.CONFIGS["c3"]
    w, qw, sc = oracle_setup(cfg)
    u = W.make_hidden(cfg)
    rng = np.random.default_rng(8)
    h0 = (rng.standard_normal((cfg.batch, cfg.d_inner, 16)) * 0.1).astype(np.float32)
    r = run_prefill(cfg, qweights_to_dev(qw), sc, u, h0=h0)
    rows, chans = _sampled(cfg, cfg.batch, cfg.seqlen, 3)
    st = check_chain(cfg, qw, sc, u, r, h0=h0, rows=rows, chans=chans)
    print("c3-layer", st)



# Taps that are copies of the library's own intermediate buffers: asking for them changes no kernel,
# so a run with them launches exactly what a call without taps (the call the benchmark times) launches:
# the row-staged GEMM epilogues and dt_proj inside the scan's first pass.
COPY_TAPS = ["u_q", "xz_q", "x_q", "dbc_q", "dt_q", "g16", "gH_q"]


@pytest.mark.parametrize("name", ["c1", "c3", "c4"])
def test_prefill_untapped_path_at_full_size(name):
    """The path `bench.py` times, at the configured shapes: (i) with the copy taps only, every link against
    the oracle (all rows at c1, sampled rows and channels at c3 / c4); (ii) with no taps at all: output and
    states are the same bits as (i); (iii) c1: the output against the oracle's own end-to-end run."""
    cfg = W.CONFIGS[name]
    w, qw, sc = oracle_setup(cfg)
    u = W.make_hidden(cfg)
    h0 = None
    if name == "c3":
        h0 = (np.random.default_rng(8).standard_normal((cfg.batch, cfg.d_inner, 16)) * 0.1).astype(np.float32)
    qd = qweights_to_dev(qw)
    r = run_prefill(cfg, qd, sc, u, h0=h0, tap_names=COPY_TAPS)
    rows, chans = (None, None) if name == "c1" else _sampled(cfg, cfg.batch, cfg.seqlen, 11)
    st = check_chain(cfg, qw, sc, u, r, h0=h0, rows=rows, chans=chans)
    r0 = run_prefill(cfg, qd, sc, u, h0=h0, taps=False)
    assert np.array_equal(r0["out"].view(np.uint16), r["out"].view(np.uint16))
    assert np.array_equal(r0["h"].view(np.uint32), r["h"].view(np.uint32))
    assert np.array_equal(r0["conv_state"].view(np.uint16), r["conv_state"].view(np.uint16))
    # the float taps switch on one more store in the scan and the Hadamard kernel, nothing else
    r1 = run_prefill(cfg, qd, sc, u, h0=h0, tap_names=COPY_TAPS + ["y_f32", "gH_f32"])
    check_chain(cfg, qw, sc, u, r1, h0=h0, rows=rows, chans=chans)
    assert np.array_equal(r1["out"].view(np.uint16), r["out"].view(np.uint16))
    if name == "c1":
        ref = O.q_prefill(qw, sc, u)
        e = end_to_end(r0, ref, name)
        assert rel_err(r0["h"], ref["h"]) <= 2e-2
        assert np.array_equal(r0["conv_state"].view(np.uint16), ref["conv_state"].view(np.uint16))
        print(name, st, "end-to-end", e)


def _decode_steps(cfg, Bt, steps, qw, sc, check_every=1, fused_dt=False):
    qd = qweights_to_dev(qw)
    ssm_np, cs_np = W.make_decode_state(cfg, batch=Bt)
    ssm, cs = dev(ssm_np), dev(cs_np)
    ws = workspace(Q.quamba_workspace_bytes(cfg, Bt, 1))
    out = empty((Bt, cfg.d_model), torch.float16)
    from gpu_util import TAP_SHAPES
    # without the raw dt_proj sums among the taps the scan step computes dt_q itself
    tp = make_taps(cfg, Bt, [n for n in TAP_SHAPES if n != "acc_dt"] if fused_dt else None)
    o_ssm, o_cs = ssm_np, cs_np
    for s in range(steps):
        u = W.make_hidden(cfg, batch=Bt, seqlen=1, stream=100 + s)
        state_before = {"ssm_state": host(ssm).copy(), "conv_state": host(cs).copy()}
        Q.quamba_mixer_decode(cfg, qd, sc, dev(u[:, 0]), Bt, out, ssm, cs, tp, ws)
        r = {k: host(v) for k, v in tp.items()}
        r["out"] = host(out)
        r["h"] = host(ssm)
        if s % check_every == 0:
            check_chain(cfg, qw, sc, u, r, decode_state=state_before)
        # the oracle's own trajectory, for the end-to-end comparison
        ref = O.q_decode(qw, sc, u[:, 0], o_ssm, o_cs)
        o_ssm, o_cs = ref["h"], ref["conv_state"]
        assert rel_err(r["out"].astype(np.float64), ref["out"][:, 0].astype(np.float64)) <= 2e-2
        assert rel_err(host(ssm), o_ssm) <= 2e-2
        new_cs = host(cs)
        assert np.array_equal(new_cs[:, :, :2].view(np.uint16), state_before["conv_state"][:, :, 1:].view(np.uint16))
        assert np.array_equal(new_cs.view(np.uint16), o_cs.view(np.uint16))


@pytest.mark.parametrize("fused_dt", [False, True])
def test_decode_tiny(fused_dt):
    cfg = W.tiny_config(name="td", d_model=64, d_inner=128, dt_rank=16, batch=3, seqlen=1, config_id=96)
    w, qw, sc = oracle_setup(cfg, randomize_bias=True, gain=4.0)
    _decode_steps(cfg, 3, 4, qw, sc, fused_dt=fused_dt)


@pytest.mark.parametrize("fused_dt", [False, True])
def test_decode_c2_shape(fused_dt):
    cfg = W.CONFIGS["c2"]
    w, qw, sc = oracle_setup(cfg)
    _decode_steps(cfg, cfg.batch, 3, qw, sc, fused_dt=fused_dt)



def test_decode_c2_200_consecutive_steps(capsys):
    """The generation workload as configured (2.8B layer, 64 sequences, consecutive steps on carried states), run
    for 200 steps: the calls without taps that the benchmark times, every 25th step with taps and checked
    link by link from the GPU's own states, every step's output against the oracle's own trajectory, and the
    drift of the carried states against the oracle's after the last step."""
    import sys
    import time
    cfg = W.CONFIGS["c2"]
    Bt, steps = cfg.batch, 200
    w, qw, sc = oracle_setup(cfg)
    qd = qweights_to_dev(qw)
    ssm_np, cs_np = W.make_decode_state(cfg, batch=Bt)
    ssm, cs = dev(ssm_np), dev(cs_np)
    ws = workspace(Q.quamba_workspace_bytes(cfg, Bt, 1))
    out = empty((Bt, cfg.d_model), torch.float16)
    from gpu_util import TAP_SHAPES
    tp = make_taps(cfg, Bt, [n for n in TAP_SHAPES if n != "acc_dt"])
    o_ssm, o_cs = ssm_np, cs_np
    worst_out, t0 = 0.0, time.time()
    for s in range(steps):
        u = W.make_hidden(cfg, batch=Bt, seqlen=1, stream=1000 + s)
        tapped = s % 25 == 0 or s == steps - 1
        if tapped:
            state_before = {"ssm_state": host(ssm).copy(), "conv_state": host(cs).copy()}
        Q.quamba_mixer_decode(cfg, qd, sc, dev(u[:, 0]), Bt, out, ssm, cs, tp if tapped else None, ws)
        if tapped:
            r = {k: host(v) for k, v in tp.items()}
            r["out"], r["h"] = host(out), host(ssm)
            check_chain(cfg, qw, sc, u, r, decode_state=state_before)
        ref = O.q_decode(qw, sc, u[:, 0], o_ssm, o_cs)
        o_ssm, o_cs = ref["h"], ref["conv_state"]
        e = rel_err(host(out).astype(np.float64), ref["out"][:, 0].astype(np.float64))
        worst_out = max(worst_out, e)
        assert e <= 2e-2, (s, e)
        if tapped:
            with capsys.disabled():
                print(f"  [c2 x 200] step {s}: output {e:.2e}, state {rel_err(host(ssm), o_ssm):.2e} of absmax vs the "
                      f"oracle's trajectory ({time.time() - t0:.0f} s)", file=sys.stderr, flush=True)
    # the conv window holds exact products of codes and one scale: the same bits unless an x_pre code flipped,
    # which the GEMM's bit-exact sums exclude
    assert np.array_equal(host(cs).view(np.uint16), o_cs.view(np.uint16))
    # the recurrent state after 200 steps: fp32 recurrence against fp64, plus the odd flipped code of x or dt
    # (one code on at most 0.1 % of the elements per step, forgotten at the rate exp(dt A))
    drift = rel_err(host(ssm), o_ssm)
    assert drift <= 1e-3, drift
    assert np.isfinite(host(ssm)).all()


@pytest.mark.parametrize("name,Bt", [("c2", 64), ("c2", 24), ("c2", 16), ("c2", 7), ("tiny", 6), ("c2", 100)])
def test_decode_without_taps_is_the_tapped_step(name, Bt):
    """The intermediates are checked link by link in the tapped runs above; without taps the step takes
    the faster epilogues (row-staged stores, the conv step inside in_proj's epilogue from staged codes).
    Both must leave exactly the same output and states."""
    cfg = W.CONFIGS[name] if name != "tiny" else W.tiny_config(name="tdn", d_model=1024, d_inner=256, dt_rank=16,
                                                                 batch=Bt, seqlen=1, config_id=98)
    w, qw, sc = oracle_setup(cfg)
    qd = qweights_to_dev(qw)
    ssm_np, cs_np = W.make_decode_state(cfg, batch=Bt)
    ws = workspace(Q.quamba_workspace_bytes(cfg, Bt, 1))
    from gpu_util import TAP_SHAPES
    res = []
    for taps in (make_taps(cfg, Bt, None), make_taps(cfg, Bt, [n for n in TAP_SHAPES if n != "acc_dt"]), None):
        ssm, cs = dev(ssm_np), dev(cs_np)
        out = empty((Bt, cfg.d_model), torch.float16)
        for s in range(2):
            u = W.make_hidden(cfg, batch=Bt, seqlen=1, stream=300 + s)
            Q.quamba_mixer_decode(cfg, qd, sc, dev(u[:, 0]), Bt, out, ssm, cs, taps, ws)
        res.append((host(out), host(ssm), host(cs)))
    for r in res[1:]:
        assert np.array_equal(r[0].view(np.uint16), res[0][0].view(np.uint16))
        assert np.array_equal(r[1].view(np.uint32), res[0][1].view(np.uint32))
        assert np.array_equal(r[2].view(np.uint16), res[0][2].view(np.uint16))


@pytest.mark.parametrize("dm,di,Bt", [(2560, 5120, 1), (2560, 5120, 3), (208, 1024, 3), (128, 1024, 2), (64, 2048, 2),
                                      (144, 3072, 3), (48, 10240, 1), (2560, 5120, 4)])
def test_decode_few_sequences_fused_tail_is_the_tapped_step(dm, di, Bt):
    """Up to three sequences without taps: the Hadamard transform and its quantization run inside the
    out_proj launch (orders 2^m, 12 * 2^m and 20 * 2^m; numbers of column groups that are and are not
    multiples of 8, which picks the workgroup-to-tile mapping; four sequences take the separate kernels
    again).  The tapped run, checked against the
    oracle link by link, takes the separate kernels; outputs, states and the transformed codes must
    be the same bits."""
    cfg = W.tiny_config(name="t1", d_model=dm, d_inner=di, dt_rank=16, batch=Bt, seqlen=1, config_id=96)
    w, qw, sc = oracle_setup(cfg, randomize_bias=True, gain=4.0)
    _decode_steps(cfg, Bt, 2, qw, sc, fused_dt=True)
    qd = qweights_to_dev(qw)
    ssm_np, cs_np = W.make_decode_state(cfg, batch=Bt)
    ws = workspace(Q.quamba_workspace_bytes(cfg, Bt, 1))
    res = []
    for taps in (make_taps(cfg, Bt, None), make_taps(cfg, Bt, ["gH_q"]), None):
        ssm, cs = dev(ssm_np), dev(cs_np)
        out = empty((Bt, cfg.d_model), torch.float16)
        for s in range(2):
            u = W.make_hidden(cfg, batch=Bt, seqlen=1, stream=310 + s)
            Q.quamba_mixer_decode(cfg, qd, sc, dev(u[:, 0]), Bt, out, ssm, cs, taps, ws)
        res.append((host(out), host(ssm), host(cs), None if taps is None else host(taps["gH_q"])))
    for r in res[1:]:
        assert np.array_equal(r[0].view(np.uint16), res[0][0].view(np.uint16))
        assert np.array_equal(r[1].view(np.uint32), res[0][1].view(np.uint32))
        assert np.array_equal(r[2].view(np.uint16), res[0][2].view(np.uint16))
    assert np.array_equal(res[1][3], res[0][3])


@pytest.mark.parametrize("Bt,di,rk", [(19, 32, 16), (33, 192, 80)])
def test_decode_many_sequences_ragged(Bt, di, rk):
    """Above 16 sequences the scan step walks groups of four sequences per workgroup with the W_dt rows in
    registers: a batch that is not a multiple of four, channels that do not fill the last workgroup, and a
    dt_rank that leaves the last 64-byte piece partly empty."""
    cfg = W.tiny_config(name="tdm", d_model=64, d_inner=di, dt_rank=rk, batch=Bt, seqlen=1, config_id=97)
    w, qw, sc = oracle_setup(cfg, randomize_bias=True, gain=4.0)
    _decode_steps(cfg, Bt, 3, qw, sc, fused_dt=True)


@pytest.mark.parametrize("Bt", [1, 2, 3, 4, 5, 8])
def test_decode_few_sequences_2p8b_width(Bt):
    """Generation with one or two sequences takes the streaming (no matrix tile) projections, more take
    matrix tiles."""
    cfg = W.CONFIGS["c2"]
    w, qw, sc = oracle_setup(cfg)
    _decode_steps(cfg, Bt, 2, qw, sc, fused_dt=(Bt % 2 == 1))


@pytest.mark.parametrize("Bt", [65, 130])
def test_decode_more_than_64_sequences_2p8b_width(Bt):
    """Beyond 64 sequences the projections leave the generation tile forms (in_proj no longer carries the conv
    step, the planner takes its prefill rules): same link-by-link checks, with and without the fused dt_proj."""
    cfg = W.CONFIGS["c2"]
    w, qw, sc = oracle_setup(cfg)
    _decode_steps(cfg, Bt, 2, qw, sc, fused_dt=(Bt % 2 == 1))


@pytest.mark.parametrize("Bt", [3, 4])
def test_decode_streaming_kernels_up_to_four_sequences(Bt):
    """The streaming kernels serve up to four sequences (by default they are used up to two, where they are
    the faster form): the same checks with the threshold raised."""
    cfg = W.CONFIGS["c2"]
    w, qw, sc = oracle_setup(cfg)
    try:
        Q.quamba_debug_set_gemv_max_rows(4)
        _decode_steps(cfg, Bt, 2, qw, sc, fused_dt=(Bt % 2 == 1))
    finally:
        Q.quamba_debug_set_gemv_max_rows(-1)


def test_prefill_then_decode_handoff():
    """State handed from prefill to decode: prefill(L) + one decode step tracks prefill(L+1)."""
    cfg = W.tiny_config(name="th", d_model=64, d_inner=128, dt_rank=16, batch=2, seqlen=33, config_id=97)
    w, qw, sc = oracle_setup(cfg, randomize_bias=True, gain=4.0)
    qd = qweights_to_dev(qw)
    u = W.make_hidden(cfg, seqlen=34)
    full = run_prefill(cfg, qd, sc, u, taps=False)
    part = run_prefill(cfg, qd, sc, u[:, :33], taps=False)
    ssm, cs = dev(part["h"]), dev(part["conv_state"])
    out = empty((2, cfg.d_model), torch.float16)
    ws = workspace(Q.quamba_workspace_bytes(cfg, 2, 1))
    Q.quamba_mixer_decode(cfg, qd, sc, dev(u[:, 33]), 2, out, ssm, cs, None, ws)
    assert rel_err(host(out).astype(np.float64), full["out"][:, 33].astype(np.float64)) <= 3e-2
    assert rel_err(host(ssm), full["h"]) <= 2e-2
    assert np.array_equal(host(cs).view(np.uint16), full["conv_state"].view(np.uint16))


def test_mixer_argument_errors():
    cfg = W.tiny_config(name="te", d_model=64, d_inner=128, dt_rank=16, batch=1, seqlen=4, config_id=98)
    w, qw, sc = oracle_setup(cfg)
    qd = qweights_to_dev(qw)
    u = dev(W.make_hidden(cfg))
    out = empty((1, 4, 64), torch.float16)
    small = workspace(256)
    with pytest.raises(Q.QuambaError) as e:
        Q.quamba_mixer_prefill(cfg, qd, sc, u, 1, 4, out, None, None, None, small)
    assert e.value.code == -3
    ws = workspace(Q.quamba_workspace_bytes(cfg, 1, 4))
    with pytest.raises(Q.QuambaError) as e:
        Q.quamba_mixer_prefill(cfg, qd, sc, u, 1, 0, out, None, None, None, ws)
    assert e.value.code == -1
    bad = W.tiny_config(name="tb", d_model=64, d_inner=112, dt_rank=16)  # 7 * 16: no Hadamard order
    assert Q.quamba_workspace_bytes(bad, 1, 4) == 0
    with pytest.raises(Q.QuambaError) as e:
        Q.quamba_mixer_decode(cfg, qd, sc, u, 1, out, None, None, None, ws)  # decode needs its state
    assert e.value.code == -1


def test_determinism():
    cfg = W.CONFIGS["c0"]
    w, qw, sc = oracle_setup(cfg)
    u = W.make_hidden(cfg)
    qd = qweights_to_dev(qw)
    a = run_prefill(cfg, qd, sc, u, taps=False)
    b = run_prefill(cfg, qd, sc, u, taps=False)
    assert np.array_equal(a["out"].view(np.uint16), b["out"].view(np.uint16))
    assert np.array_equal(a["h"], b["h"])


# ------------------------------------------------------------------ calibration on the GPU
@pytest.mark.parametrize("name", ["tiny", "c0"])
def test_calibrate_matches_oracle(name):
    cfg = (W.tiny_config(name="tc", d_model=64, d_inner=192, dt_rank=16, config_id=99) if name == "tiny"
           else W.CONFIGS[name])
    w = W.make_weights(cfg, randomize_bias=True)
    calib = W.make_calibration(cfg)
    p = 99.9 if name == "tiny" else 99.999
    qw_ref, sc_ref = O.calibrate(w, calib, p)
    fw = {k: dev(v) for k, v in w.items()}
    out_q = {k: torch.zeros(v.shape, dtype=torch.int8 if v.dtype == np.int8 else torch.float32, device="cuda:0")
             for k, v in qw_ref.items()}
    nb, Lc = calib.shape[:2]
    ws = workspace(Q.quamba_calibrate_workspace_bytes(cfg, nb, Lc))
    sc = Q.scales_to_dict(Q.quamba_calibrate(cfg, fw, dev(calib), nb, Lc, p, out_q, ws))
    for k in Q.SCALE_FIELDS:
        tol = 2e-3 if k in ("s_x", "inv_s_x", "m_x_dt", "m_x_B", "m_x_C") else 1e-4
        assert abs(sc[k] - float(sc_ref[k])) <= tol * abs(float(sc_ref[k])), (k, sc[k], float(sc_ref[k]))
    for k, v in qw_ref.items():
        got = host(out_q[k])
        if v.dtype == np.int8:
            d = np.abs(got.astype(int) - v.astype(int))
            assert d.max() <= 1 and (d != 0).mean() <= 1e-3, k
        else:
            assert np.array_equal(got, v), k


def test_calibrate_with_mse_clip_matches_oracle():
    """Section 5.1, enhanced variant: the scale of the scan input from the model-optimal clipping
    scalar instead of the percentile; every other scale is the one the percentile run gives."""
    cfg = W.tiny_config(name="tc", d_model=64, d_inner=192, dt_rank=16, config_id=99)
    w = W.make_weights(cfg, randomize_bias=True)
    calib = W.make_calibration(cfg)
    qw_ref, sc_ref = O.calibrate(w, calib, x_clip="mse")
    _, sc_pct = O.calibrate(w, calib)
    assert float(sc_ref["s_x"]) != float(sc_pct["s_x"])
    fw = {k: dev(v) for k, v in w.items()}
    out_q = {k: torch.zeros(v.shape, dtype=torch.int8 if v.dtype == np.int8 else torch.float32, device="cuda:0")
             for k, v in qw_ref.items()}
    nb, Lc = calib.shape[:2]
    ws = workspace(Q.quamba_calibrate_workspace_bytes(cfg, nb, Lc))
    sc = Q.scales_to_dict(Q.quamba_calibrate_x_rule(cfg, fw, dev(calib), nb, Lc, Q.X_MSE_CLIP, 99.999, out_q, ws))
    for k in Q.SCALE_FIELDS:
        # x on the GPU is an fp32 forward, the oracle's an fp64 one: the clip moves with the few values near it
        tol = 2e-3 if k in ("s_x", "inv_s_x", "m_x_dt", "m_x_B", "m_x_C") else 1e-4
        assert abs(sc[k] - float(sc_ref[k])) <= tol * abs(float(sc_ref[k])), (k, sc[k], float(sc_ref[k]))
    with pytest.raises(Q.QuambaError):
        Q.quamba_calibrate_x_rule(cfg, fw, dev(calib), nb, Lc, 7, 99.999, out_q, ws)


@pytest.mark.parametrize("name", ["tiny", "c0"])
def test_fp32_mixer_matches_oracle(name):
    """The unquantized mixer of Section 3.1 on the GPU (fp32) against the oracle's fp64 one."""
    cfg = W.tiny_config(name="tf", d_model=64, d_inner=192, dt_rank=16, config_id=98) if name == "tiny" else W.CONFIGS[name]
    w = W.make_weights(cfg, randomize_bias=True)
    nb, L = (3, 37) if name == "tiny" else (2, 130)
    u = W.make_hidden(cfg, batch=nb, seqlen=L, stream=11)
    want = O.fp_forward(w, u)["out"].reshape(nb * L, cfg.d_model)
    fw = {k: dev(v) for k, v in w.items()}
    out = empty((nb * L, cfg.d_model), torch.float32)
    Q.quamba_mixer_fp32(cfg, fw, dev(u), nb, L, out, workspace(Q.quamba_calibrate_workspace_bytes(cfg, nb, L)))
    assert rel_err(host(out), want) <= 1e-4
    with pytest.raises(Q.QuambaError):
        Q.quamba_mixer_fp32(cfg, fw, dev(u), nb, L, out, workspace(1024))


def test_x_scale_rules_rank_as_in_the_oracle():
    """Table "percentiles": error of the quantized mixer against the unquantized one for the
    percentile sweep and the clipping optimisation, on weights whose scan input has a few
    far-reaching channels (no outlier channels in the hidden input, so x decides the error).
    The whole GPU pipeline (calibration, quantized prefill, fp32 reference) must reproduce the
    oracle's error for every rule, and with it the shape of the sweep."""
    import dataclasses
    cfg = dataclasses.replace(W.CONFIGS["c0"], name="c0x", config_id=77, outlier_gain=1.0)
    w = W.make_weights(cfg, x_outlier_rows=8, x_outlier_gain=8.0)
    calib = W.make_calibration(cfg)
    nb, Lc = calib.shape[:2]
    L = 128
    u = W.make_hidden(cfg, batch=1, seqlen=L, stream=5)
    ref_o = O.fp_forward(w, u)["out"].reshape(L, cfg.d_model)
    fw = {k: dev(v) for k, v in w.items()}
    ref_g = empty((L, cfg.d_model), torch.float32)
    Q.quamba_mixer_fp32(cfg, fw, dev(u), 1, L, ref_g, workspace(Q.quamba_calibrate_workspace_bytes(cfg, 1, L)))
    ref_g = host(ref_g).astype(np.float64)
    ws = workspace(Q.quamba_calibrate_workspace_bytes(cfg, nb, Lc))
    err_o, err_g = {}, {}
    for rule in (99.0, 99.99, 100.0, "mse"):
        qw_o, sc_o = (O.calibrate(w, calib, x_clip="mse") if rule == "mse" else O.calibrate(w, calib, rule))
        out_o = O.q_prefill(qw_o, sc_o, u)["out"].reshape(L, cfg.d_model).astype(np.float64)
        err_o[rule] = np.linalg.norm(out_o - ref_o) / np.linalg.norm(ref_o)
        out_q = {k: torch.zeros(v.shape, dtype=torch.int8 if v.dtype == np.int8 else torch.float32, device="cuda:0")
                 for k, v in qw_o.items()}
        sc_g = Q.scales_to_dict(Q.quamba_calibrate_x_rule(
            cfg, fw, dev(calib), nb, Lc, Q.X_MSE_CLIP if rule == "mse" else Q.X_PERCENTILE,
            99.999 if rule == "mse" else rule, out_q, ws))
        got = run_prefill(cfg, out_q, sc_g, u, taps=False)["out"].reshape(L, cfg.d_model).astype(np.float64)
        err_g[rule] = np.linalg.norm(got - ref_g) / np.linalg.norm(ref_g)
    for rule in err_o:
        assert err_g[rule] == pytest.approx(err_o[rule], rel=0.03), (rule, err_g, err_o)
    assert err_g[99.0] > 1.5 * err_g[99.99] and err_g[100.0] > 1.1 * err_g[99.99]
    assert err_g["mse"] <= 1.05 * min(err_g[99.0], err_g[99.99], err_g[100.0])


def test_misaligned_weights_and_states_are_refused():
    """The kernels read weights in 16-byte pieces and the states in 16- / 8-byte pieces: a pointer
    that does not allow it is an argument error, not a fault."""
    cfg = W.tiny_config(name="tm", d_model=64, d_inner=128, dt_rank=16, config_id=88)
    w, qw, sc = oracle_setup(cfg)
    u = dev(W.make_hidden(cfg, batch=1, seqlen=8))
    out = empty((1, 8, cfg.d_model), torch.float16)
    ws = workspace(Q.quamba_workspace_bytes(cfg, 1, 8))
    for key in ("W_in", "W_x", "W_outH", "conv_w"):
        qd = qweights_to_dev(qw)
        shifted = torch.zeros(qd[key].numel() + 16, dtype=torch.int8, device="cuda:0")
        shifted[1:1 + qd[key].numel()] = qd[key].reshape(-1)
        qd[key] = shifted[1:1 + qd[key].numel()]  # one byte off a 16-byte boundary
        with pytest.raises(Q.QuambaError):
            Q.quamba_mixer_prefill(cfg, qd, sc, u, 1, 8, out, None, None, None, ws)
    qd = qweights_to_dev(qw)
    ssm = torch.zeros(cfg.d_inner * cfg.d_state + 4, dtype=torch.float32, device="cuda:0")[1:1 + cfg.d_inner * cfg.d_state]
    with pytest.raises(Q.QuambaError):
        Q.quamba_mixer_prefill(cfg, qd, sc, u, 1, 8, out, ssm, None, None, ws)
    Q.quamba_mixer_prefill(cfg, qd, sc, u, 1, 8, out, None, None, None, ws)  # the aligned call still works


def test_two_calls_in_flight_on_two_streams():
    """Calls that share no output, state or workspace may overlap on different streams: each must
    give what it gives alone."""
    cfg = W.CONFIGS["c0"]
    w, qw, sc = oracle_setup(cfg)
    qd = qweights_to_dev(qw)
    us = [dev(W.make_hidden(cfg, batch=2, seqlen=300, stream=40 + i)) for i in range(2)]
    alone = []
    for u in us:
        out = empty((2, 300, cfg.d_model), torch.float16)
        ssm = torch.zeros((2, cfg.d_inner, cfg.d_state), dtype=torch.float32, device="cuda:0")
        Q.quamba_mixer_prefill(cfg, qd, sc, u, 2, 300, out, ssm, None, None, workspace(Q.quamba_workspace_bytes(cfg, 2, 300)))
        torch.cuda.synchronize()
        alone.append((host(out), host(ssm)))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [empty((2, 300, cfg.d_model), torch.float16) for _ in range(2)]
    ssms = [torch.zeros((2, cfg.d_inner, cfg.d_state), dtype=torch.float32, device="cuda:0") for _ in range(2)]
    wss = [workspace(Q.quamba_workspace_bytes(cfg, 2, 300)) for _ in range(2)]
    torch.cuda.synchronize()
    for rep in range(6):  # several rounds so that the two streams really interleave
        for i in range(2):
            with torch.cuda.stream(streams[i]):
                if rep:
                    ssms[i].zero_()  # h0 = 0 again, ordered on the call's own stream
                Q.quamba_mixer_prefill(cfg, qd, sc, us[i], 2, 300, outs[i], ssms[i], None, None, wss[i], streams[i])
    torch.cuda.synchronize()
    for i in range(2):
        assert np.array_equal(host(outs[i]).view(np.uint16), alone[i][0].view(np.uint16))
        assert np.array_equal(host(ssms[i]), alone[i][1])


@pytest.mark.parametrize("path", ["static", "dynamic_x"])
def test_decode_steps_replayed_from_a_hip_graph(path):
    """The decode call enqueues kernel launches only, so a caller may capture it.  Several replays,
    with eager work and synchronisations in between, must each reproduce the eager result bit for bit.
    (dynamic_x: the variant that forms the scale of x on the device; its word for the maximum is cleared
    by a kernel, so it captures as well.)"""
    cfg = W.tiny_config(name="tg", d_model=64, d_inner=128, dt_rank=16, batch=3, seqlen=1, config_id=89)
    w, qw, sc = oracle_setup(cfg, randomize_bias=True, gain=4.0)
    qd = qweights_to_dev(qw)
    Bt, nsteps = 3, 4
    us = dev(np.stack([W.make_hidden(cfg, batch=Bt, seqlen=1, stream=300 + s)[:, 0] for s in range(nsteps)]))
    ssm0_np, cs0_np = W.make_decode_state(cfg, batch=Bt)
    dyn = path == "dynamic_x"
    ws = workspace(Q.quamba_xdyn_workspace_bytes(cfg, Bt, 1) if dyn else Q.quamba_workspace_bytes(cfg, Bt, 1))
    outs = empty((nsteps, Bt, cfg.d_model), torch.float16)
    ssm, cs = dev(ssm0_np), dev(cs0_np)
    qs, scs, dims = Q.make_qweights(qd), Q.scales_from_dict(sc), Q.make_dims(cfg)

    def steps():
        for s in range(nsteps):
            if dyn:
                Q.quamba_mixer_decode_xdyn(dims, qs, scs, us[s], Bt, outs[s], ssm, cs, None, None, None, ws,
                                           torch.cuda.current_stream())
            else:
                Q.quamba_mixer_decode(dims, qs, scs, us[s], Bt, outs[s], ssm, cs, None, ws, torch.cuda.current_stream())

    steps()  # eager reference (also the warm-up that sets kernel attributes outside the capture)
    ref_out, ref_ssm, ref_cs = host(outs).copy(), host(ssm).copy(), host(cs).copy()

    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    ssm.copy_(dev(ssm0_np)); cs.copy_(dev(cs0_np))
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=cap):
        steps()
    for rep in range(3):
        ssm.copy_(dev(ssm0_np)); cs.copy_(dev(cs0_np)); outs.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(host(outs).view(np.uint16), ref_out.view(np.uint16)), rep
        assert np.array_equal(host(ssm), ref_ssm), rep
        assert np.array_equal(host(cs).view(np.uint16), ref_cs.view(np.uint16)), rep
        # eager work between the replays
        ssm.copy_(dev(ssm0_np)); cs.copy_(dev(cs0_np))
        steps()
        torch.cuda.synchronize()
        assert np.array_equal(host(outs).view(np.uint16), ref_out.view(np.uint16))
