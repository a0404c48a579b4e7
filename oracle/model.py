"""Whole-model shell around the stack of Quamba blocks (oracle side; test infrastructure).

What the paper times as time to first token, time per output token and time to last token
(Section 5.2) is the full language model: token embedding, the stack of blocks (residual add +
RMSNorm + quantization, quantized mixer: Section 4.3), a final residual add + RMSNorm, the
output head and greedy selection of the next token.  The embedding and the head stay in half
precision (Section 4.3 quantizes the blocks only) and share one matrix, as in the Mamba models
the paper quantizes.

    res_{-1} = E[token]  (fp16),  out_{-1} = 0
    block l:  (u_q, res_l) = add_rmsnorm_quant(out_{l-1}, res_{l-1});  out_l = mixer_l(u_q)
    y = RMSNorm(out_{last} + res_{last}) * w_f   (fp16),   logits = y E^T,   next = argmax logits

A model is a dict: E fp16 [V, Dm], norm_f fp16 [Dm], norm_w list of fp16 [Dm], layers list of
(qw, sc) as returned by ``calibrate``, eps.  The states of generation are, per layer, the fp32
recurrent state [Bt, Di, N] and the fp16 conv window [Bt, Di, 3].
"""
from __future__ import annotations

import numpy as np

from .stack import q_stack_decode, q_stack_prefill

F32 = np.float32
F64 = np.float64


def embed(E, tokens):
    """Rows of the embedding matrix: fp16 [..., Dm]."""
    return np.asarray(E, dtype=np.float16)[np.asarray(tokens)]


def final_norm(out, res, weight, eps=1e-5):
    """fp16(RMSNorm(out + res) * weight); the sum is rounded to fp16 first, like every residual."""
    s = (np.asarray(out).astype(F32) + np.asarray(res).astype(F32)).astype(np.float16)
    r = s.astype(F64)
    ms = np.mean(r * r, axis=-1, keepdims=True)
    return (r / np.sqrt(ms + eps) * np.asarray(weight).astype(F64)).astype(np.float16)


def lm_head(y, E):
    """logits[b, v] = sum_k y[b, k] E[v, k], fp64 sums of the fp16 values."""
    return np.asarray(y).astype(F64) @ np.asarray(E).astype(F64).T


def greedy(logits):
    """Index of the largest logit per row; the lowest index among equal maxima."""
    return np.argmax(np.asarray(logits), axis=-1).astype(np.int32)


def model_prefill(model, tokens):
    """tokens int [Bt, L] -> (logits fp64 [Bt, V] of the last position, next token [Bt], states)."""
    hidden = embed(model["E"], tokens)
    trace, out, res = q_stack_prefill(model["layers"], model["norm_w"], hidden, model["eps"])
    y = final_norm(out[:, -1, :], res[:, -1, :], model["norm_f"], model["eps"])
    logits = lm_head(y, model["E"])
    states = [(p["t"]["h"], p["t"]["conv_state"]) for p in trace]
    return logits, greedy(logits), states


def model_decode(model, tokens, states):
    """One generation step: tokens int [Bt] -> (logits, next token, new states)."""
    hidden = embed(model["E"], tokens)
    _, out, res, new_states = q_stack_decode(model["layers"], model["norm_w"], hidden, states, model["eps"])
    y = final_norm(out, res, model["norm_f"], model["eps"])
    logits = lm_head(y, model["E"])
    return logits, greedy(logits), new_states


def model_generate(model, prompt, n_new):
    """Greedy generation: prefill the prompt [Bt, L], then n_new - 1 decode steps.
    Returns int32 [Bt, n_new] (the tokens after the prompt) and the logits of every step."""
    logits, nxt, states = model_prefill(model, prompt)
    toks, all_logits = [nxt], [logits]
    for _ in range(n_new - 1):
        logits, nxt, states = model_decode(model, nxt, states)
        toks.append(nxt)
        all_logits.append(logits)
    return np.stack(toks, axis=1), all_logits
