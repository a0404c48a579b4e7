"""The 64-block configuration (Mamba-2.8B width, batch 4) as a whole chain on the GPU against the oracle.

The sequences are shortened (4 x 64 tokens, then 8 generation steps) so that the oracle's 64 calibrations and
its own pass over the stack finish in a few minutes; widths, depth, batch and per-layer static scales are the
configuration's.  Three kinds of check:

  * links: the same chain issued block by block through the stage entry points (residual add + RMSNorm +
    quantizer, quantized mixer) gives every block's input and output; on blocks 0, 1, 31 and 63 each stage is
    compared with the oracle's stage function applied to the GPU's own input of that stage;
  * identity: `quamba_model_prefill` / `quamba_model_decode` must leave exactly the bits of that block-by-block
    chain in all 64 recurrent states, all 64 conv windows and the logits (any aliasing of the residual buffers
    or of the shared workspace across blocks would break this);
  * end to end: logits and states against the oracle's own run of the whole model.
"""
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle as O
import paper_2410_13229_amd as Q
import workloads as W
from gpu_util import assert_lsb, dev, empty, host, make_taps, qweights_to_dev, rel_err, workspace
from test_gpu_mixer import COPY_TAPS, check_chain

pytestmark = pytest.mark.gpu

NLAYERS, BT, L, STEPS, VOCAB = 64, 4, 64, 8, 4096
LINKS = (0, 1, 31, 63)
TAPS = COPY_TAPS + ["y_f32", "gH_f32"]


def _say(capsys, msg):
    with capsys.disabled():
        print(msg, file=sys.stderr, flush=True)


def _lazy_weights(cfg, n):
    """Yields the fp32 weights of layer 0, 1, ... while a helper thread draws the next ones."""
    with ThreadPoolExecutor(max_workers=1) as ex:
        nxt = ex.submit(W.make_weights, cfg, 0)
        for l in range(n):
            w = nxt.result()
            if l + 1 < n:
                nxt = ex.submit(W.make_weights, cfg, l + 1)
            yield w


def _bits_equal(a, b):
    return torch.equal(a.contiguous().view(torch.uint8), b.contiguous().view(torch.uint8))


def test_c3_64_blocks_prefill_then_decode(capsys):
    cfg = W.CONFIGS["c3"]
    Dm, Di = cfg.d_model, cfg.d_inner
    t0 = time.time()
    # token embedding = seeded hidden vectors of the configuration's recipe (N(0,1), 4 channels x 50)
    E = W.make_hidden(cfg, batch=1, seqlen=VOCAB, stream=9)[0]
    norm_w, norm_f = W.make_norm_weights(cfg, NLAYERS)
    calib = O.embed(E, W.make_tokens(cfg, VOCAB, batch=4, seqlen=64, stream=7))

    class Progress:  # calibrate_stack walks this once; tells the log where it is
        def __iter__(self):
            for l, w in enumerate(_lazy_weights(cfg, NLAYERS)):
                if l % 8 == 0:
                    _say(capsys, f"  [c3 stack] oracle calibration, layer {l} ({time.time() - t0:.0f} s)")
                yield w

    layers = O.calibrate_stack(Progress(), norm_w, calib)
    assert len(layers) == NLAYERS
    om = dict(E=E, norm_f=norm_f, norm_w=norm_w, layers=layers, eps=1e-5)
    qds = [qweights_to_dev(qw) for qw, _ in layers]
    dn = [dev(nw) for nw in norm_w]
    dE, dnf = dev(E), dev(norm_f)
    gm = Q.make_model(cfg, dE, dnf, [(qd, sc, nw) for qd, (_, sc), nw in zip(qds, layers, dn)], eps=1e-5)
    prompt = W.make_tokens(cfg, VOCAB, batch=BT, seqlen=L)
    _say(capsys, f"  [c3 stack] oracle prefill over 64 blocks ({time.time() - t0:.0f} s)")
    hidden = O.embed(E, prompt)
    ref_trace, ref_out, ref_res = O.q_stack_prefill(layers, norm_w, hidden)
    ref_logits = O.lm_head(O.final_norm(ref_out[:, -1], ref_res[:, -1], norm_f, 1e-5), E)
    ref_states = [(p["t"]["h"], p["t"]["conv_state"]) for p in ref_trace]
    for p in ref_trace:  # keep only what the checks below read
        p["t"] = {"out": p["t"]["out"]}

    # ---- prefill, block by block through the stage entry points
    _say(capsys, f"  [c3 stack] GPU prefill: block-by-block chain and links ({time.time() - t0:.0f} s)")
    M = BT * L
    wsb = workspace(Q.quamba_workspace_bytes(cfg, BT, L))
    dtok = dev(prompt)
    res = empty((BT, L, Dm), torch.float16)
    out = empty((BT, L, Dm), torch.float16)
    u_q = empty((BT, L, Dm), torch.int8)
    Q.quamba_embed(dE, dtok, M, Dm, VOCAB, res, out)
    assert np.array_equal(host(res).view(np.uint16), hidden.view(np.uint16))
    ssm_c = torch.zeros((NLAYERS, BT, Di, 16), dtype=torch.float32, device="cuda:0")
    cs_c = empty((NLAYERS, BT, Di, 3), torch.float16)
    for l, (qw, sc) in enumerate(layers):
        link = l in LINKS
        if link:
            out_in, res_in = host(out).copy(), host(res).copy()
        Q.quamba_add_rmsnorm_quant(out, res, dn[l], 1e-5, sc["inv_s_u"], u_q, M, Dm)
        tp = make_taps(cfg, M, TAPS) if link else None
        Q.quamba_mixer_prefill_q(cfg, qds[l], sc, u_q, BT, L, out, ssm_c[l], cs_c[l], tp, wsb)
        if link:
            uq_ref, res_ref = O.add_rmsnorm_quant(out_in, res_in, norm_w[l], sc["inv_s_u"], 1e-5)
            assert np.array_equal(host(res).view(np.uint16), res_ref.view(np.uint16)), l
            assert_lsb(host(u_q), uq_ref, f"u_q of block {l}")
            r = {k: host(v) for k, v in tp.items()}
            r["out"], r["h"] = host(out), host(ssm_c[l])
            u_deq = (host(u_q).astype(np.float32) * np.float32(sc["s_u"])).astype(np.float16)
            assert np.array_equal(O.quantize(u_deq.astype(np.float32), sc["inv_s_u"]), r["u_q"].reshape(BT, L, Dm))
            check_chain(cfg, qw, sc, u_deq, r)
            # the residual stream and the block output against the oracle's own chain, this deep
            e_res = rel_err(host(res).astype(np.float64), ref_trace[l]["res"].astype(np.float64))
            e_out = rel_err(host(out).astype(np.float64), ref_trace[l]["t"]["out"].astype(np.float64))
            _say(capsys, f"  [c3 stack] block {l}: residual {e_res:.2e}, output {e_out:.2e} of absmax vs the oracle's chain")
            assert e_res <= 5e-2 and e_out <= 1e-1, (l, e_res, e_out)
    y_c = empty((BT, Dm), torch.float16)
    Q.quamba_final_norm(out, res, dnf, 1e-5, BT, L, Dm, y_c)
    logits_c = empty((BT, VOCAB), torch.float32)
    Q.quamba_lm_head(y_c, dE, BT, VOCAB, Dm, logits_c)

    # ---- the same prefill through the model entry point: the same bits everywhere
    ssm = torch.full((NLAYERS, BT, Di, 16), 7.0, dtype=torch.float32, device="cuda:0")
    cs = empty((NLAYERS, BT, Di, 3), torch.float16)
    logits = empty((BT, VOCAB), torch.float32)
    nxt = empty((BT,), torch.int32)
    Q.quamba_model_prefill(gm, dtok, BT, L, logits, nxt, ssm, cs, workspace(Q.quamba_model_workspace_bytes(gm, BT, L)))
    torch.cuda.synchronize()
    assert _bits_equal(ssm, ssm_c) and _bits_equal(cs, cs_c) and _bits_equal(logits, logits_c)
    assert np.array_equal(host(nxt), O.greedy(host(logits)))
    e = rel_err(host(logits), ref_logits)
    _say(capsys, f"  [c3 stack] prefill logits vs the oracle's own run: {e:.2e} of absmax")
    assert e <= 5e-2
    for l in LINKS:
        assert rel_err(host(ssm[l]), ref_states[l][0]) <= 5e-2, l
        assert rel_err(host(cs[l]).astype(np.float64), ref_states[l][1].astype(np.float64)) <= 5e-2, l

    # ---- generation steps on the carried states
    wsd = workspace(Q.quamba_model_workspace_bytes(gm, BT, 1))
    wsm = workspace(Q.quamba_workspace_bytes(cfg, BT, 1))
    dres, dout, duq = empty((BT, Dm), torch.float16), empty((BT, Dm), torch.float16), empty((BT, Dm), torch.int8)
    tok = O.greedy(ref_logits)
    for step in range(STEPS):
        _say(capsys, f"  [c3 stack] generation step {step} ({time.time() - t0:.0f} s)")
        dtk = dev(tok)
        ssm_c, cs_c = ssm.clone(), cs.clone()
        full_oracle = step in (0, STEPS - 1)
        st_in = [(host(ssm[l]).copy(), host(cs[l]).copy()) for l in range(NLAYERS)] if full_oracle else None
        # block by block
        Q.quamba_embed(dE, dtk, BT, Dm, VOCAB, dres, dout)
        for l, (qw, sc) in enumerate(layers):
            link = l in LINKS
            if link:
                out_in, res_in = host(dout).copy(), host(dres).copy()
                state_in = {"ssm_state": host(ssm_c[l]).copy(), "conv_state": host(cs_c[l]).copy()}
            Q.quamba_add_rmsnorm_quant(dout, dres, dn[l], 1e-5, sc["inv_s_u"], duq, BT, Dm)
            tp = make_taps(cfg, BT, TAPS) if link else None
            Q.quamba_mixer_decode_q(cfg, qds[l], sc, duq, BT, dout, ssm_c[l], cs_c[l], tp, wsm)
            if link:
                uq_ref, res_ref = O.add_rmsnorm_quant(out_in, res_in, norm_w[l], sc["inv_s_u"], 1e-5)
                assert np.array_equal(host(dres).view(np.uint16), res_ref.view(np.uint16)), (step, l)
                assert_lsb(host(duq), uq_ref, f"u_q of block {l}, step {step}", frac=2e-3)  # 10 k elements: 0.1 % = 10
                r = {k: host(v) for k, v in tp.items()}
                r["out"], r["h"] = host(dout), host(ssm_c[l])
                u_deq = (host(duq).astype(np.float32) * np.float32(sc["s_u"])).astype(np.float16)[:, None, :]
                check_chain(cfg, qw, sc, u_deq, r, decode_state=state_in)
        Q.quamba_final_norm(dout, dres, dnf, 1e-5, BT, 1, Dm, y_c)
        Q.quamba_lm_head(y_c, dE, BT, VOCAB, Dm, logits_c)
        # the model entry point from the same states
        Q.quamba_model_decode(gm, dtk, BT, logits, nxt, ssm, cs, wsd)
        torch.cuda.synchronize()
        assert _bits_equal(ssm, ssm_c) and _bits_equal(cs, cs_c), step
        assert _bits_equal(logits, logits_c), step
        assert np.array_equal(host(nxt), O.greedy(host(logits)))
        if full_oracle:  # the oracle's whole model from the GPU's states of this step
            o_logits, _, o_states = O.model_decode(om, tok, st_in)
            e = rel_err(host(logits), o_logits)
            _say(capsys, f"  [c3 stack] step {step} logits vs the oracle's model step: {e:.2e} of absmax")
            assert e <= 5e-2, (step, e)
            for l in LINKS:
                assert rel_err(host(ssm[l]), o_states[l][0]) <= 5e-2, (step, l)
                assert np.array_equal(host(cs[l])[:, :, :2].view(np.uint16), st_in[l][1][:, :, 1:].view(np.uint16))
        tok = host(nxt).copy()
