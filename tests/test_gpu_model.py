"""GPU parity of the whole-model shell: embedding, block stack, final norm, tied head, greedy
selection, generation on carried states (eager and replayed from a HIP graph)."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2410_13229_amd as Q
import workloads as W
from gpu_util import dev, empty, host, qweights_to_dev, rel_err, workspace

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------ the shell's own stages
@pytest.mark.parametrize("M,Dm,vocab", [(1, 64, 5), (37, 96, 97), (300, 2560, 1000)])
def test_embed_rows_bit_exact_and_out_cleared(M, Dm, vocab):
    rng = np.random.default_rng(M + Dm)
    E = (rng.standard_normal((vocab, Dm)) * 0.02).astype(np.float16)
    tok = rng.integers(0, vocab, M, dtype=np.int32)
    tok[0] = vocab - 1
    if M > 2:
        tok[1], tok[2] = -7, vocab + 3  # out of range: clamped
    res = torch.full((M, Dm), 3.0, dtype=torch.float16, device="cuda:0")
    out = torch.full((M, Dm), 3.0, dtype=torch.float16, device="cuda:0")
    Q.quamba_embed(dev(E), dev(tok), M, Dm, vocab, res, out)
    want = O.embed(E, np.clip(tok, 0, vocab - 1))
    assert np.array_equal(host(res).view(np.uint16), want.view(np.uint16))
    assert not host(out).any()


@pytest.mark.parametrize("Bt,L,Dm", [(1, 1, 64), (3, 5, 96), (4, 17, 2560), (2, 3, 8192)])
def test_final_norm_last_positions(Bt, L, Dm):
    rng = np.random.default_rng(Bt * 100 + L + Dm)
    out = rng.standard_normal((Bt, L, Dm)).astype(np.float16)
    res = (rng.standard_normal((Bt, L, Dm)) * 3).astype(np.float16)
    w = (1 + 0.1 * rng.standard_normal(Dm)).astype(np.float16)
    y = empty((Bt, Dm), torch.float16)
    Q.quamba_final_norm(dev(out), dev(res), dev(w), 1e-5, Bt, L, Dm, y)
    want = O.final_norm(out[:, -1], res[:, -1], w, 1e-5).astype(np.float64)
    got = host(y).astype(np.float64)
    # fp32 arithmetic then one rounding to fp16, against fp64 then one rounding: one fp16 ulp at most
    assert np.abs(got - want).max() <= 2.0 ** -10 * np.maximum(np.abs(want), 2.0 ** -14).max()
    assert (np.abs(got - want) > 2.0 ** -10 * np.abs(want) + 1e-7).mean() == 0.0


@pytest.mark.parametrize("Bt,V,Dm", [(1, 5, 64), (2, 97, 64), (64, 1000, 96), (70, 50280, 2560), (3, 1003, 768)])
def test_lm_head_and_argmax(Bt, V, Dm):
    rng = np.random.default_rng(Bt + V + Dm)
    y = rng.standard_normal((Bt, Dm)).astype(np.float16)
    E = (rng.standard_normal((V, Dm)) * 0.02).astype(np.float16)
    logits = torch.full((Bt, V), -5.0, dtype=torch.float32, device="cuda:0")
    dE = dev(E)
    Q.quamba_lm_head(dev(y), dE, Bt, V, Dm, logits)
    want = O.lm_head(y, E)
    assert rel_err(host(logits), want) <= 1e-5  # fp32 sums of exact fp16 products
    nxt = empty((Bt,), torch.int32)
    Q.quamba_argmax(logits, Bt, V, nxt)
    assert np.array_equal(host(nxt), O.greedy(host(logits)))


def test_argmax_lowest_index_among_equal_maxima():
    V = 1000
    lg = np.full((3, V), -1.0, dtype=np.float32)
    lg[0, [700, 300, 999]] = 4.0
    lg[1, :] = 2.0
    lg[2, 999] = 0.5
    nxt = empty((3,), torch.int32)
    Q.quamba_argmax(dev(lg), 3, V, nxt)
    assert host(nxt).tolist() == [300, 0, 999]


# ------------------------------------------------------------------ the model
def _tiny_model(nlayers, config_id, vocab, gain=4.0, d_model=64, d_inner=128):
    cfg = W.tiny_config(name="gm", d_model=d_model, d_inner=d_inner, dt_rank=16, batch=2, seqlen=12,
                        config_id=config_id, n_outlier=1, outlier_gain=8.0)
    ws = []
    for l in range(nlayers):
        w = W.make_weights(cfg, layer=l, randomize_bias=True)
        for k in ("W_in", "conv_w", "W_x", "W_dt", "W_out"):
            w[k] = w[k] * np.float32(gain)
        ws.append(w)
    norm_w, norm_f = W.make_norm_weights(cfg, nlayers)
    E = W.make_embedding(cfg, vocab)
    calib = O.embed(E, W.make_tokens(cfg, vocab, batch=4, seqlen=32, stream=7))
    layers = O.calibrate_stack(ws, norm_w, calib)
    om = dict(E=E, norm_f=norm_f, norm_w=norm_w, layers=layers, eps=1e-5)
    gm = Q.make_model(cfg, dev(E), dev(norm_f),
                      [(qweights_to_dev(qw), sc, dev(nw)) for (qw, sc), nw in zip(layers, norm_w)], eps=1e-5)
    return cfg, om, gm


def _states(cfg, nlayers, Bt):
    ssm = torch.full((nlayers, Bt, cfg.d_inner, 16), 7.0, dtype=torch.float32, device="cuda:0")  # prefill clears it
    cs = empty((nlayers, Bt, cfg.d_inner, 3), torch.float16)
    return ssm, cs


def _check_choice(next_gpu, logits_oracle, tol):
    """The chosen token is the oracle's, or its oracle logit is within tol of the oracle's maximum."""
    top = logits_oracle.max(axis=-1)
    chosen = logits_oracle[np.arange(len(next_gpu)), next_gpu]
    assert np.all(chosen >= top - tol), (next_gpu, O.greedy(logits_oracle), top - chosen)


@pytest.mark.parametrize("nlayers,Bt,L,vocab", [(2, 2, 12, 97), (3, 1, 45, 256), (1, 3, 1, 1000)])
def test_model_prefill_then_decode_steps(nlayers, Bt, L, vocab):
    cfg, om, gm = _tiny_model(nlayers, 97 + nlayers, vocab)
    prompt = W.make_tokens(cfg, vocab, batch=Bt, seqlen=L)
    ws = workspace(Q.quamba_model_workspace_bytes(gm, Bt, L))
    ssm, cs = _states(cfg, nlayers, Bt)
    logits = empty((Bt, vocab), torch.float32)
    nxt = empty((Bt,), torch.int32)
    Q.quamba_model_prefill(gm, dev(prompt), Bt, L, logits, nxt, ssm, cs, ws)
    ref_logits, ref_next, ref_states = O.model_prefill(om, prompt)
    scale = np.abs(ref_logits).max()
    assert rel_err(host(logits), ref_logits) <= 5e-2
    assert np.array_equal(host(nxt), O.greedy(host(logits)))  # the selection itself is exact
    _check_choice(host(nxt), ref_logits, 0.1 * scale)
    for l in range(nlayers):
        assert rel_err(host(ssm[l]), ref_states[l][0]) <= 5e-2
        assert rel_err(host(cs[l]).astype(np.float64), ref_states[l][1].astype(np.float64)) <= 5e-2
    # two steps on the carried states, each fed the oracle's own previous choice and checked against
    # the oracle run from the GPU's states (a link check: errors do not compound)
    wsd = workspace(Q.quamba_model_workspace_bytes(gm, Bt, 1))
    tok = ref_next
    for step in range(2):
        st_in = [(host(ssm[l]).copy(), host(cs[l]).copy()) for l in range(nlayers)]
        Q.quamba_model_decode(gm, dev(tok), Bt, logits, nxt, ssm, cs, wsd)
        ref_logits, ref_next, ref_states = O.model_decode(om, tok, st_in)
        assert rel_err(host(logits), ref_logits) <= 5e-2, step
        _check_choice(host(nxt), ref_logits, 0.1 * np.abs(ref_logits).max())
        for l in range(nlayers):
            assert rel_err(host(ssm[l]), ref_states[l][0]) <= 5e-2
        tok = ref_next


def test_model_generate_eager_and_graph_agree_with_each_other_and_track_the_oracle():
    nlayers, Bt, L, vocab, n_new = 2, 2, 12, 97, 6
    cfg, om, gm = _tiny_model(nlayers, 99, vocab)
    prompt = W.make_tokens(cfg, vocab, batch=Bt, seqlen=L)
    wsp = workspace(Q.quamba_model_workspace_bytes(gm, Bt, L))
    wsd = workspace(Q.quamba_model_workspace_bytes(gm, Bt, 1))
    first = empty((Bt,), torch.int32)
    side = torch.cuda.Stream()
    runs = []
    # eager, graph, some unrelated eager work, graph again, eager again: every run must give the same tokens
    for use_graph in (False, True, True, False):
        ssm, cs = _states(cfg, nlayers, Bt)
        Q.quamba_model_prefill(gm, dev(prompt), Bt, L, None, first, ssm, cs, wsp)
        torch.cuda.synchronize()
        toks = torch.full((n_new, Bt), -1, dtype=torch.int32, device="cuda:0")
        with torch.cuda.stream(side):
            Q.quamba_model_generate(gm, first, Bt, n_new, toks, ssm, cs, wsd, use_graph=use_graph, stream=side)
        side.synchronize()
        runs.append((host(first).copy(), host(toks).copy(), host(ssm).copy()))
        junk = torch.randn(1 << 16, device="cuda:0")
        (junk * 2).sum().item()
    for f, t, s in runs[1:]:
        assert np.array_equal(f, runs[0][0]) and np.array_equal(t, runs[0][1])
        assert np.array_equal(s, runs[0][2])
    assert (runs[0][1] >= 0).all() and (runs[0][1] < vocab).all()
    # against the oracle: walk the GPU's own token sequence through the oracle and require every GPU choice
    # to be (near-)maximal for the oracle's logits at that step
    first_gpu, toks_gpu, _ = runs[0]
    ref_logits, _, states = O.model_prefill(om, prompt)
    _check_choice(first_gpu, ref_logits, 0.1 * np.abs(ref_logits).max())
    tok = first_gpu
    for i in range(n_new):
        ref_logits, _, states = O.model_decode(om, tok, states)
        _check_choice(toks_gpu[i], ref_logits, 0.1 * np.abs(ref_logits).max())
        tok = toks_gpu[i]


@pytest.mark.parametrize("Bt,d_model,d_inner", [(1, 96, 192), (3, 96, 192), (8, 96, 192), (2, 5120, 10240)])
def test_few_sequence_generation_kernels_match_the_general_path(Bt, d_model, d_inner):
    """With at most 8 sequences a block's norm, in_proj and conv step run in one kernel; the general path
    (separate kernels, matrix tiles) must give the same step up to the odd code that flips because the two
    sum the squares of a row in a different order."""
    # (d_model 5120: a row no longer fits the one-sweep form of the fused kernel's normalisation)
    nlayers, vocab = (2, 256) if d_model < 1000 else (1, 64)
    cfg, om, gm = _tiny_model(nlayers, 101, vocab, d_model=d_model, d_inner=d_inner)
    prompt = W.make_tokens(cfg, vocab, batch=Bt, seqlen=9)
    wsp = workspace(Q.quamba_model_workspace_bytes(gm, Bt, 9))
    wsd = workspace(Q.quamba_model_workspace_bytes(gm, Bt, 1))
    res = []
    try:
        Q.quamba_debug_set_gemv_max_rows(4)  # the few-row kernels up to the 4 rows they serve (default: 2)
        for fuse in (1, 0):
            Q.quamba_debug_set_fuse_decode(fuse)
            ssm, cs = _states(cfg, nlayers, Bt)
            nxt = empty((Bt,), torch.int32)
            Q.quamba_model_prefill(gm, dev(prompt), Bt, 9, None, nxt, ssm, cs, wsp)
            logits = empty((Bt, vocab), torch.float32)
            steps = []
            for _ in range(3):
                Q.quamba_model_decode(gm, nxt, Bt, logits, nxt, ssm, cs, wsd)
                steps.append((host(logits).copy(), host(ssm).copy(), host(cs).copy()))
            res.append(steps)
    finally:
        Q.quamba_debug_set_fuse_decode(1)
        Q.quamba_debug_set_gemv_max_rows(-1)
    for (la, sa, ca), (lb, sb, cb) in zip(*res):
        assert rel_err(la, lb) <= 2e-2
        assert rel_err(sa, sb) <= 2e-2
        assert (ca.view(np.uint16) != cb.view(np.uint16)).mean() <= 2e-3


@pytest.mark.parametrize("Bt,d_model,d_inner", [(24, 256, 512), (64, 256, 512), (7, 512, 1024), (3, 256, 512), (4, 512, 1024)])
def test_many_sequence_generation_fusions_are_the_general_path_bit_for_bit(Bt, d_model, d_inner):
    """With more than 2 sequences the projections whose K is split over the grid hand their partial sums to
    the kernel that follows (x_proj to the scan step, out_proj to the next block's add + norm + quantization)
    instead of a reduce kernel.  Integer sums, the same roundings: logits, states and tokens must be the same
    bits as with the separate kernels."""
    nlayers, vocab = 3, 128
    cfg, om, gm = _tiny_model(nlayers, 103, vocab, d_model=d_model, d_inner=d_inner)
    prompt = W.make_tokens(cfg, vocab, batch=Bt, seqlen=5)
    wsp = workspace(Q.quamba_model_workspace_bytes(gm, Bt, 5))
    wsd = workspace(Q.quamba_model_workspace_bytes(gm, Bt, 1))
    res = []
    try:
        for fuse in (1, 0):
            Q.quamba_debug_set_fuse_decode(fuse)
            ssm, cs = _states(cfg, nlayers, Bt)
            nxt = empty((Bt,), torch.int32)
            Q.quamba_model_prefill(gm, dev(prompt), Bt, 5, None, nxt, ssm, cs, wsp)
            logits = empty((Bt, vocab), torch.float32)
            steps = []
            for _ in range(3):
                Q.quamba_model_decode(gm, nxt, Bt, logits, nxt, ssm, cs, wsd)
                steps.append((host(logits).copy(), host(ssm).copy(), host(cs).copy(), host(nxt).copy()))
            res.append(steps)
    finally:
        Q.quamba_debug_set_fuse_decode(1)
    for (la, sa, ca, ta), (lb, sb, cb, tb) in zip(*res):
        assert np.array_equal(la.view(np.uint32), lb.view(np.uint32))
        assert np.array_equal(sa.view(np.uint32), sb.view(np.uint32))
        assert np.array_equal(ca.view(np.uint16), cb.view(np.uint16))
        assert np.array_equal(ta, tb)


def test_model_rejects_bad_arguments():
    cfg, om, gm = _tiny_model(1, 100, 97)
    ws = workspace(Q.quamba_model_workspace_bytes(gm, 1, 4))
    ssm, cs = _states(cfg, 1, 1)
    tok = dev(np.zeros((1, 4), dtype=np.int32))
    with pytest.raises(Q.QuambaError):
        Q.quamba_model_prefill(gm, tok, 1, 4, None, None, ssm, cs, workspace(256))  # workspace too small
    with pytest.raises(Q.QuambaError):
        Q.quamba_model_prefill(gm, None, 1, 4, None, None, ssm, cs, ws)
    with pytest.raises(Q.QuambaError):
        Q.quamba_model_generate(gm, tok, 1, 3, empty((3, 1), torch.int32), ssm, cs, ws, use_graph=True, stream=0)
    assert Q.quamba_model_workspace_bytes(gm, 0, 4) == 0


# ------------------------------------------------------------------ per-layer calibration of a stack
def test_calibrate_block_chain_matches_oracle_stack_calibration():
    nlayers = 3
    cfg = W.tiny_config(name="gc", d_model=64, d_inner=128, dt_rank=16, batch=2, seqlen=12, config_id=102,
                        n_outlier=1, outlier_gain=8.0)
    ws_np = []
    for l in range(nlayers):
        w = W.make_weights(cfg, layer=l, randomize_bias=True)
        for k in ("W_in", "conv_w", "W_x", "W_dt", "W_out"):
            w[k] = w[k] * np.float32(4.0)
        ws_np.append(w)
    norm_w, _ = W.make_norm_weights(cfg, nlayers)
    hidden = W.make_calibration(cfg)
    nb, Lc = hidden.shape[:2]
    ref = O.calibrate_stack(ws_np, norm_w, hidden)
    res = dev(hidden.astype(np.float32).reshape(nb * Lc, -1))
    out = torch.zeros_like(res)
    wsb = workspace(Q.quamba_calibrate_workspace_bytes(cfg, nb, Lc))
    for l in range(nlayers):
        qw_ref, sc_ref = ref[l]
        out_q = {k: torch.zeros(v.shape, dtype=torch.int8 if v.dtype == np.int8 else torch.float32, device="cuda:0")
                 for k, v in qw_ref.items()}
        sc = Q.scales_to_dict(Q.quamba_calibrate_block(cfg, {k: dev(v) for k, v in ws_np[l].items()}, dev(norm_w[l]),
                                                       1e-5, res, out, nb, Lc, 99.999, out_q, wsb))
        for k in Q.SCALE_FIELDS:
            tol = 2e-3 if k in ("s_x", "inv_s_x", "m_x_dt", "m_x_B", "m_x_C") else 2e-4
            assert abs(sc[k] - float(sc_ref[k])) <= tol * abs(float(sc_ref[k])), (l, k, sc[k], float(sc_ref[k]))
        for k, v in qw_ref.items():
            got = host(out_q[k])
            if v.dtype == np.int8:
                d = np.abs(got.astype(int) - v.astype(int))
                assert d.max() <= 1 and (d != 0).mean() <= 1e-3, (l, k)
            else:
                assert np.array_equal(got, v), (l, k)


def test_model_two_blocks_at_2p8b_width_and_full_vocabulary():
    """The 64-block configuration's width (d_model 2560, d_inner 5120, dt_rank 160) and vocabulary (50280) with two
    blocks, batch 4: prefill, then generation steps on the few-sequence kernels, against the oracle."""
    cfg = W.CONFIGS["c3"]
    nlayers, Bt, L, vocab = 2, 4, 48, 50280
    ws_np = [W.make_weights(cfg, layer=l) for l in range(nlayers)]
    norm_w, norm_f = W.make_norm_weights(cfg, nlayers)
    E = W.make_embedding(cfg, vocab)
    calib = O.embed(E, W.make_tokens(cfg, vocab, batch=2, seqlen=128, stream=7))
    layers = O.calibrate_stack(ws_np, norm_w, calib)
    om = dict(E=E, norm_f=norm_f, norm_w=norm_w, layers=layers, eps=1e-5)
    gm = Q.make_model(cfg, dev(E), dev(norm_f),
                      [(qweights_to_dev(qw), sc, dev(nw)) for (qw, sc), nw in zip(layers, norm_w)], eps=1e-5)
    prompt = W.make_tokens(cfg, vocab, batch=Bt, seqlen=L)
    ssm, cs = _states(cfg, nlayers, Bt)
    logits = empty((Bt, vocab), torch.float32)
    nxt = empty((Bt,), torch.int32)
    Q.quamba_model_prefill(gm, dev(prompt), Bt, L, logits, nxt, ssm, cs,
                           workspace(Q.quamba_model_workspace_bytes(gm, Bt, L)))
    ref_logits, ref_next, ref_states = O.model_prefill(om, prompt)
    assert rel_err(host(logits), ref_logits) <= 5e-2
    assert np.array_equal(host(nxt), O.greedy(host(logits)))
    _check_choice(host(nxt), ref_logits, 0.1 * np.abs(ref_logits).max())
    for l in range(nlayers):
        assert rel_err(host(ssm[l]), ref_states[l][0]) <= 5e-2
    wsd = workspace(Q.quamba_model_workspace_bytes(gm, Bt, 1))
    tok = ref_next
    for step in range(2):
        st_in = [(host(ssm[l]).copy(), host(cs[l]).copy()) for l in range(nlayers)]
        Q.quamba_model_decode(gm, dev(tok), Bt, logits, nxt, ssm, cs, wsd)
        ref_logits, ref_next, ref_states = O.model_decode(om, tok, st_in)
        assert rel_err(host(logits), ref_logits) <= 5e-2, step
        _check_choice(host(nxt), ref_logits, 0.1 * np.abs(ref_logits).max())
        for l in range(nlayers):
            assert rel_err(host(ssm[l]), ref_states[l][0]) <= 5e-2
        tok = ref_next
