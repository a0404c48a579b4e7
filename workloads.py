"""Seeded synthetic inputs for the W8A8 Mamba-mixer workloads.

This module only *draws numbers*: it holds none of the method's arithmetic (no
quantizer, no scan, no Hadamard).  Both the CPU oracle's tests and the HIP path's
tests/bench take their inputs from here, so the two sides see the same bytes.

The tensors stand in for the trained Mamba / Jamba checkpoints and the Pile
calibration sentences the paper used (Section 5.1, "Model and datasets" and
"Quantization setup"); they take the paper's layer *shapes* and a value recipe with
a few large-magnitude hidden channels, not its data.

All draws are counter-based: ``Philox(key=[SEED, 1000*config_id + tensor_id])`` so
every tensor is reproducible on its own, in any order.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED = 241013229


@dataclass(frozen=True)
class MixerConfig:
    """Shape of one Mamba mixer plus the workload run on it."""

    name: str
    config_id: int
    d_model: int
    d_inner: int
    d_state: int
    dt_rank: int
    d_conv: int
    batch: int
    seqlen: int
    n_outlier: int
    outlier_gain: float
    calib_batch: int = 4
    calib_len: int = 256


CONFIGS = {
    # Mamba-130M layer, batch 1, L=256
    "c0": MixerConfig("c0", 0, 768, 1536, 16, 48, 4, 1, 256, 4, 50.0),
    # Mamba-2.8B layer, batch 1, L=2048 prefill
    "c1": MixerConfig("c1", 1, 2560, 5120, 16, 160, 4, 1, 2048, 4, 50.0),
    # Mamba-2.8B layer, decode, batch 64, L=1
    "c2": MixerConfig("c2", 2, 2560, 5120, 16, 160, 4, 64, 1, 4, 50.0),
    # Mamba-2.8B stack (64 layers), batch 4, L=4096
    "c3": MixerConfig("c3", 3, 2560, 5120, 16, 160, 4, 4, 4096, 4, 50.0, 4, 512),
    # Jamba-shaped Mamba layer, batch 1, L=16384
    "c4": MixerConfig("c4", 4, 4096, 8192, 16, 256, 4, 1, 16384, 8, 100.0),
}

# tensor ids (the low part of the Philox key)
_T_W_IN, _T_CONV_W, _T_W_X, _T_W_DT, _T_W_OUT, _T_DT_BIAS = 1, 2, 3, 4, 5, 6
_T_OUTLIER_IDX, _T_CALIB, _T_HIDDEN, _T_SSM_STATE, _T_CONV_STATE = 10, 11, 12, 13, 14
_T_CONV_B, _T_D = 15, 16
_T_EMBED, _T_NORM, _T_TOKENS = 20, 21, 22
_T_X_ROWS = 23


def tiny_config(name="tiny", d_model=64, d_inner=128, dt_rank=16, batch=2, seqlen=37,
                config_id=90, n_outlier=2, outlier_gain=50.0):
    """A small configuration for brute-force checks (d_state = 16, conv width 4)."""
    return MixerConfig(name, config_id, d_model, d_inner, 16, dt_rank, 4, batch, seqlen,
                       n_outlier, outlier_gain, 2, 32)


def _rng(cfg: MixerConfig, tensor_id: int, layer: int = 0, stream: int = 0):
    key = [SEED, (cfg.config_id * 1000 + tensor_id) + (layer << 20) + (stream << 40)]
    return np.random.Generator(np.random.Philox(key=key))


def make_weights(cfg: MixerConfig, layer: int = 0, randomize_bias: bool = False,
                 x_outlier_rows: int = 0, x_outlier_gain: float = 1.0):
    """fp32 master weights of one mixer.

    W_in [2*Di, Dm] (rows [0,Di) produce x, rows [Di,2Di) produce z), conv_w [Di, W],
    conv_b [Di], W_x [R+2N, Di] (rows dt | B | C), W_dt [Di, R], dt_bias [Di],
    A_log [Di, N], D [Di], W_out [Dm, Di].

    Dense and conv weights are N(0, 0.02^2); A_log[d, n] = log(n+1); D = 1 and
    conv_b = 0 unless ``randomize_bias`` (unit tests) draws them; dt_bias is the
    inverse softplus of a log-uniform time step in [1e-3, 1e-1].

    ``x_outlier_rows`` > 0 multiplies that many seeded rows of the x half of W_in by
    ``x_outlier_gain``: a few channels of the scan input then reach well beyond the rest, the
    situation Section 4.2 describes for x (rare, moderately large values), which is what the
    choice of clipping rule for x is evaluated on.
    """
    Dm, Di, N, R, W = cfg.d_model, cfg.d_inner, cfg.d_state, cfg.dt_rank, cfg.d_conv
    std = 0.02

    def normal(tid, shape):
        return (_rng(cfg, tid, layer).standard_normal(shape, dtype=np.float32) * np.float32(std))

    w = {
        "W_in": normal(_T_W_IN, (2 * Di, Dm)),
        "conv_w": normal(_T_CONV_W, (Di, W)),
        "W_x": normal(_T_W_X, (R + 2 * N, Di)),
        "W_dt": normal(_T_W_DT, (Di, R)),
        "W_out": normal(_T_W_OUT, (Dm, Di)),
    }
    if x_outlier_rows > 0:
        rows = _rng(cfg, _T_X_ROWS, layer).choice(Di, size=x_outlier_rows, replace=False)
        w["W_in"][np.sort(rows)] *= np.float32(x_outlier_gain)
    u = _rng(cfg, _T_DT_BIAS, layer).random(Di)
    dt = np.exp(u * (np.log(1e-1) - np.log(1e-3)) + np.log(1e-3))
    w["dt_bias"] = (dt + np.log(-np.expm1(-dt))).astype(np.float32)
    w["A_log"] = np.tile(np.log(np.arange(1, N + 1, dtype=np.float64)), (Di, 1)).astype(np.float32)
    if randomize_bias:
        w["conv_b"] = (_rng(cfg, _T_CONV_B, layer).standard_normal(Di, dtype=np.float32)
                       * np.float32(0.1))
        w["D"] = (_rng(cfg, _T_D, layer).standard_normal(Di, dtype=np.float32)
                  * np.float32(0.5) + np.float32(1.0))
    else:
        w["conv_b"] = np.zeros(Di, dtype=np.float32)
        w["D"] = np.ones(Di, dtype=np.float32)
    return w


def outlier_channels(cfg: MixerConfig, layer: int = 0):
    """Indices of the hidden channels that carry the large-magnitude values."""
    idx = _rng(cfg, _T_OUTLIER_IDX, layer).choice(cfg.d_model, size=cfg.n_outlier, replace=False)
    return np.sort(idx)


def _hidden(cfg, tensor_id, shape, layer, stream):
    h = _rng(cfg, tensor_id, layer, stream).standard_normal(shape, dtype=np.float32)
    h[..., outlier_channels(cfg, layer)] *= np.float32(cfg.outlier_gain)
    return h.astype(np.float16)


def make_calibration(cfg: MixerConfig, layer: int = 0):
    """fp16 calibration batch [calib_batch, calib_len, Dm] (same outlier channels as the
    test inputs, a different value stream)."""
    return _hidden(cfg, _T_CALIB, (cfg.calib_batch, cfg.calib_len, cfg.d_model), layer, 0)


def make_hidden(cfg: MixerConfig, batch=None, seqlen=None, layer: int = 0, stream: int = 0):
    """fp16 hidden input [batch, seqlen, Dm]: N(0,1) with the outlier channels scaled."""
    b = cfg.batch if batch is None else batch
    l = cfg.seqlen if seqlen is None else seqlen
    return _hidden(cfg, _T_HIDDEN, (b, l, cfg.d_model), layer, stream)


def make_decode_state(cfg: MixerConfig, batch=None, layer: int = 0):
    """Carried decode state: ssm_state fp32 [B, Di, N] ~ N(0, 0.1^2); conv_state fp16
    [B, Di, W-1] ~ N(0, 2.2^2) (about the spread of the conv input under this recipe)."""
    b = cfg.batch if batch is None else batch
    ssm = _rng(cfg, _T_SSM_STATE, layer).standard_normal((b, cfg.d_inner, cfg.d_state),
                                                         dtype=np.float32) * np.float32(0.1)
    conv = _rng(cfg, _T_CONV_STATE, layer).standard_normal((b, cfg.d_inner, cfg.d_conv - 1),
                                                           dtype=np.float32) * np.float32(2.2)
    return ssm, conv.astype(np.float16)


# ------------------------------------------------------------------ whole-model shell inputs
def make_embedding(cfg: MixerConfig, vocab: int):
    """fp16 token embedding [vocab, Dm] ~ N(0, 0.02^2) (also the output head: tied)."""
    e = _rng(cfg, _T_EMBED).standard_normal((vocab, cfg.d_model), dtype=np.float32) * np.float32(0.02)
    return e.astype(np.float16)


def make_norm_weights(cfg: MixerConfig, n_layers: int):
    """RMSNorm weights: n_layers block norms and the final norm, fp16 [Dm] ~ 1 + 0.1 N(0,1)."""
    rng = _rng(cfg, _T_NORM)
    ws = [(1.0 + 0.1 * rng.standard_normal(cfg.d_model, dtype=np.float32)).astype(np.float16)
          for _ in range(n_layers + 1)]
    return ws[:-1], ws[-1]


def make_tokens(cfg: MixerConfig, vocab: int, batch=None, seqlen=None, stream: int = 0):
    """int32 token ids [batch, seqlen], uniform over the vocabulary."""
    b = cfg.batch if batch is None else batch
    l = cfg.seqlen if seqlen is None else seqlen
    return _rng(cfg, _T_TOKENS, 0, stream).integers(0, vocab, (b, l), dtype=np.int32)
