"""Pins for the oracle's multi-layer composition (Section 4.3 "Fused RMSNorm")."""
import numpy as np

import oracle as O
import workloads as W


def _stack(cfg, nlayers, gain=4.0):
    ws = []
    for l in range(nlayers):
        w = W.make_weights(cfg, layer=l, randomize_bias=True)
        for k in ("W_in", "conv_w", "W_x", "W_dt", "W_out"):
            w[k] = w[k] * np.float32(gain)
        ws.append(w)
    rng = np.random.default_rng(3)
    nws = [(1 + 0.1 * rng.standard_normal(cfg.d_model)).astype(np.float16) for _ in range(nlayers)]
    return ws, nws


def test_stack_residual_stream_and_per_layer_scales():
    cfg = W.tiny_config(name="ts", d_model=64, d_inner=128, dt_rank=16, batch=2, seqlen=24, config_id=93,
                        n_outlier=1, outlier_gain=8.0)
    ws, nws = _stack(cfg, 3)
    layers = O.calibrate_stack(ws, nws, W.make_calibration(cfg))
    hidden = W.make_hidden(cfg)
    trace, out, res = O.q_stack_prefill(layers, nws, hidden)
    # layer 0 normalises the input itself; the residual stream accumulates the block outputs in fp16
    assert np.array_equal(trace[0]["res"].view(np.uint16), hidden.view(np.uint16))
    want = hidden
    for l in range(1, 3):
        want = (trace[l - 1]["t"]["out"].astype(np.float32) + want.astype(np.float32)).astype(np.float16)
        assert np.array_equal(trace[l]["res"].view(np.uint16), want.view(np.uint16))
    assert np.array_equal(res.view(np.uint16), want.view(np.uint16))
    # every layer's input scale maps the calibration absmax of its own normalised input to 127
    assert len({float(sc["s_u"]) for _, sc in layers}) == 3
    for l in range(3):
        u_q = trace[l]["u_q"]
        assert u_q.dtype == np.int8 and np.abs(u_q.astype(int)).max() >= 64


def test_stack_prefill_then_decode_tracks_longer_prefill():
    cfg = W.tiny_config(name="ts2", d_model=64, d_inner=128, dt_rank=16, batch=2, seqlen=20, config_id=94,
                        n_outlier=1, outlier_gain=8.0)
    ws, nws = _stack(cfg, 2)
    layers = O.calibrate_stack(ws, nws, W.make_calibration(cfg))
    hidden = W.make_hidden(cfg, seqlen=21)
    full, out_full, _ = O.q_stack_prefill(layers, nws, hidden)
    part, _, _ = O.q_stack_prefill(layers, nws, hidden[:, :20])
    states = [(p["t"]["h"], p["t"]["conv_state"]) for p in part]
    _, out1, _, _ = O.q_stack_decode(layers, nws, hidden[:, 20], states)
    ref = out_full[:, 20].astype(np.float64)
    assert np.abs(out1.astype(np.float64) - ref).max() <= 0.06 * np.abs(ref).max()
