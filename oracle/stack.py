"""A stack of Quamba blocks (oracle side; test infrastructure): residual add + RMSNorm + static
quantization between quantized mixers (Section 4.3 "Fused RMSNorm"), for the multi-layer
configuration.  Block l:  (u_q, res) = add_rmsnorm_quant(out_{l-1}, res_{l-1});  out_l = mixer_l(u_q)
with out_{-1} = 0 and res_{-1} = the fp16 hidden input, so res_0 is the input itself."""
from __future__ import annotations

import numpy as np

from .mixer import add_rmsnorm_quant, calibrate, fp_forward, q_decode, q_prefill

F64 = np.float64


def _rmsnorm_fp(r, weight, eps):
    ms = np.mean(r * r, axis=-1, keepdims=True)
    return r / np.sqrt(ms + eps) * np.asarray(weight, dtype=F64)


def calibrate_stack(weights, norm_weights, calib_hidden, x_percentile=99.999, eps=1e-5):
    """Per-layer static scales (Section 5.1): layer l is calibrated on the unquantized forward of the
    layers before it.  weights: list of fp32 weight dicts; norm_weights: list of fp16 [Dm] vectors;
    calib_hidden fp16 [nb, Lc, Dm].  Returns a list of (qw, sc)."""
    res = np.asarray(calib_hidden, dtype=F64)
    out = np.zeros_like(res)
    layers = []
    for w, nw in zip(weights, norm_weights):
        res = out + res
        u = _rmsnorm_fp(res, nw, eps)
        layers.append(calibrate(w, u, x_percentile))
        out = fp_forward(w, u)["out"]
    return layers


def q_stack_prefill(layers, norm_weights, hidden, eps=1e-5):
    """Quantized stack over whole sequences.  Returns per-layer dicts (u_q, res, mixer taps) and
    the final (out, res) pair."""
    res = np.asarray(hidden, dtype=np.float16)
    out = np.zeros_like(res)
    trace = []
    for (qw, sc), nw in zip(layers, norm_weights):
        u_q, res = add_rmsnorm_quant(out, res, nw, sc["inv_s_u"], eps)
        t = q_prefill(qw, sc, u_q=u_q)
        out = t["out"]
        trace.append(dict(u_q=u_q, res=res, t=t))
    return trace, out, res


def q_stack_decode(layers, norm_weights, hidden, states, eps=1e-5):
    """One generation step through the stack.  hidden fp16 [Bt, Dm]; states: list of
    (ssm_state, conv_state) per layer.  Returns (trace, out, res, new_states)."""
    res = np.asarray(hidden, dtype=np.float16)
    out = np.zeros_like(res)
    trace, new_states = [], []
    for ((qw, sc), nw), (ssm, cs) in zip(zip(layers, norm_weights), states):
        u_q, res = add_rmsnorm_quant(out, res, nw, sc["inv_s_u"], eps)
        t = q_decode(qw, sc, None, ssm, cs, u_q=u_q)
        out = t["out"][:, 0]
        trace.append(dict(u_q=u_q, res=res, t=t))
        new_states.append((t["h"], t["conv_state"]))
    return trace, out, res, new_states
