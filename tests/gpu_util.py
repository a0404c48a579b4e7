"""Helpers for the GPU parity tests: device buffers via torch, calls via the C ABI binding."""
import numpy as np
import torch

import oracle as O
import paper_2410_13229_amd as Q
import workloads as W

DEV = "cuda:0"


def dev(a):
    """numpy array -> contiguous device tensor with the same bits."""
    a = np.ascontiguousarray(a)
    return torch.from_numpy(a).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


def empty(shape, dtype):
    return torch.empty(shape, dtype=dtype, device=DEV)


def workspace(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=DEV)


def lsb_stats(got, want):
    """(max abs code difference, fraction of elements that differ)."""
    d = np.abs(got.astype(np.int32) - want.astype(np.int32))
    return int(d.max()) if d.size else 0, float((d != 0).mean()) if d.size else 0.0


def assert_lsb(got, want, name, frac=1e-3):
    """Requantized int8 tensors may differ by <= 1 LSB on <= 0.1 % of the elements."""
    mx, fr = lsb_stats(got, want)
    assert mx <= 1, f"{name}: max code difference {mx}"
    assert fr <= frac, f"{name}: {fr:.2e} of the elements differ"


def rel_err(got, want):
    """max |got - want| / max |want| (error normalised by the tensor's absmax)."""
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    den = np.abs(want).max()
    return float(np.abs(got - want).max() / (den if den > 0 else 1.0))


_CACHE = {}


def oracle_setup(cfg, randomize_bias=False, gain=1.0):
    """(weights, qw, sc) of one layer from the oracle's calibration, cached per config."""
    key = (cfg.name, cfg.d_model, cfg.d_inner, cfg.dt_rank, randomize_bias, gain)
    if key not in _CACHE:
        w = W.make_weights(cfg, randomize_bias=randomize_bias)
        if gain != 1.0:
            for k in ("W_in", "conv_w", "W_x", "W_dt", "W_out"):
                w[k] = w[k] * np.float32(gain)
        qw, sc = O.calibrate(w, W.make_calibration(cfg))
        _CACHE[key] = (w, qw, sc)
    return _CACHE[key]


def qweights_to_dev(qw):
    return {k: dev(v) for k, v in qw.items()}


TAP_SHAPES = {
    "u_q": ("Dm", torch.int8), "acc_in": ("2Di", torch.int32), "xz_q": ("2Di", torch.int8),
    "x_q": ("Di", torch.int8), "acc_x": ("NX", torch.int32), "dbc_q": ("NX", torch.int8),
    "acc_dt": ("Di", torch.int32), "dt_q": ("Di", torch.int8), "y_f32": ("Di", torch.float32),
    "g16": ("Di", torch.float16), "gH_f32": ("Di", torch.float32), "gH_q": ("Di", torch.int8),
    "acc_out": ("Dm", torch.int32),
}


def make_taps(cfg, M, names=None):
    cols = {"Dm": cfg.d_model, "Di": cfg.d_inner, "2Di": 2 * cfg.d_inner,
            "NX": cfg.dt_rank + 2 * cfg.d_state}
    names = TAP_SHAPES.keys() if names is None else names
    return {n: empty((M, cols[TAP_SHAPES[n][0]]), TAP_SHAPES[n][1]) for n in names}


def run_prefill(cfg, qw_d, sc, u, h0=None, want_state=True, taps=True, u_q=None, tap_names=None):
    """Call quamba_mixer_prefill(_q); returns dict(out, h, conv_state, taps...) as numpy."""
    Bt, L = (u if u is not None else u_q).shape[:2]
    M = Bt * L
    ws = workspace(Q.quamba_workspace_bytes(cfg, Bt, L))
    out = empty((Bt, L, cfg.d_model), torch.float16)
    ssm = None
    if want_state:
        ssm = dev(h0) if h0 is not None else torch.zeros((Bt, cfg.d_inner, cfg.d_state), dtype=torch.float32,
                                                         device=DEV)
    cs = empty((Bt, cfg.d_inner, cfg.d_conv - 1), torch.float16)
    tp = make_taps(cfg, M, tap_names) if taps else None
    if u_q is None:
        Q.quamba_mixer_prefill(cfg, qw_d, sc, dev(u), Bt, L, out, ssm, cs, tp, ws)
    else:
        Q.quamba_mixer_prefill_q(cfg, qw_d, sc, dev(u_q), Bt, L, out, ssm, cs, tp, ws)
    r = {"out": host(out), "conv_state": host(cs)}
    if ssm is not None:
        r["h"] = host(ssm)
    if tp:
        r.update({k: host(v) for k, v in tp.items()})
    return r
