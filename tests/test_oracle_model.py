"""Pins for the oracle's whole-model shell (embedding, stack, final norm, tied head, greedy
selection; the quantities Section 5.2 times are steps of this loop)."""
import numpy as np

import oracle as O
import workloads as W

VOCAB = 97


def _model(nlayers=2, config_id=95, gain=4.0):
    cfg = W.tiny_config(name="tm", d_model=64, d_inner=128, dt_rank=16, batch=2, seqlen=12, config_id=config_id,
                        n_outlier=1, outlier_gain=8.0)
    ws = []
    for l in range(nlayers):
        w = W.make_weights(cfg, layer=l, randomize_bias=True)
        for k in ("W_in", "conv_w", "W_x", "W_dt", "W_out"):
            w[k] = w[k] * np.float32(gain)
        ws.append(w)
    norm_w, norm_f = W.make_norm_weights(cfg, nlayers)
    E = W.make_embedding(cfg, VOCAB)
    calib = O.embed(E, W.make_tokens(cfg, VOCAB, batch=4, seqlen=32, stream=7))
    layers = O.calibrate_stack(ws, norm_w, calib)
    return cfg, dict(E=E, norm_f=norm_f, norm_w=norm_w, layers=layers, eps=1e-5)


def test_embed_picks_rows_and_head_of_one_hot_is_a_column():
    cfg, m = _model(1)
    tok = np.array([[3, 96, 0], [5, 5, 42]])
    h = O.embed(m["E"], tok)
    assert h.dtype == np.float16 and h.shape == (2, 3, 64)
    assert np.array_equal(h[0, 1], m["E"][96]) and np.array_equal(h[1, 0], h[1, 1])
    y = np.zeros((1, 64), dtype=np.float16)
    y[0, 17] = 2.0
    assert np.array_equal(O.lm_head(y, m["E"])[0], 2.0 * m["E"][:, 17].astype(np.float64))


def test_final_norm_closed_form_and_greedy_ties():
    w = np.linspace(0.5, 1.5, 64).astype(np.float16)
    c = np.float16(3.0)
    out = np.full((2, 64), c / 2, dtype=np.float16)
    y = O.final_norm(out, out, w, eps=1e-5)  # every element of the sum is c: rms = |c|
    want = (w.astype(np.float64) * 3.0 / np.sqrt(9.0 + 1e-5)).astype(np.float16)
    assert np.array_equal(y[0], want) and np.array_equal(y[1], want)
    # scale invariance up to eps, sign symmetry
    big = O.final_norm(out * 8, out * 8, w, eps=0.0).astype(np.float64)
    assert np.allclose(big, O.final_norm(out, out, w, eps=0.0).astype(np.float64), rtol=2e-3)
    assert np.array_equal(O.final_norm(-out, -out, w), -y)
    assert np.array_equal(O.greedy(np.array([[1.0, 5.0, 5.0, 2.0], [7.0, 0.0, 7.0, 7.0]])), [1, 0])


def test_generation_by_carried_state_tracks_prefill_of_the_grown_sequence():
    """The recurrent route (prefill once, then one step per token on the carried states) and the
    parallel route (prefill of prompt + generated tokens) are the same function of the tokens; the
    two differ only through the decode form of the conv, which works on a dequantized window."""
    cfg, m = _model(2)
    prompt = W.make_tokens(cfg, VOCAB, batch=2, seqlen=12)
    toks, logits = O.model_generate(m, prompt, 4)
    assert toks.shape == (2, 4) and toks.dtype == np.int32
    assert np.array_equal(toks[:, 0], O.greedy(logits[0]))
    grown = prompt
    for i in range(4):
        ref_logits, ref_next, _ = O.model_prefill(m, grown)
        err = np.abs(logits[i] - ref_logits).max() / np.abs(ref_logits).max()
        assert err <= 0.08, (i, err)
        grown = np.concatenate([grown, toks[:, i:i + 1]], axis=1)
    # the first step has no decode in it: identical
    l0, n0, _ = O.model_prefill(m, prompt)
    assert np.array_equal(l0, logits[0]) and np.array_equal(n0, toks[:, 0])


def test_states_returned_by_prefill_are_the_last_layer_states():
    cfg, m = _model(2, config_id=96)
    prompt = W.make_tokens(cfg, VOCAB, batch=2, seqlen=9)
    _, _, states = O.model_prefill(m, prompt)
    assert len(states) == 2
    for ssm, cs in states:
        assert ssm.shape == (2, 128, 16) and ssm.dtype == np.float32
        assert cs.shape == (2, 128, 3) and cs.dtype == np.float16
    # a prompt that differs only in its last token leaves the conv windows' older two entries alone
    p2 = prompt.copy()
    p2[:, -1] = (p2[:, -1] + 1) % VOCAB
    _, _, s2 = O.model_prefill(m, p2)
    assert np.array_equal(states[0][1][..., :2], s2[0][1][..., :2])
    assert not np.array_equal(states[0][1][..., 2], s2[0][1][..., 2])
