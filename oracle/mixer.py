"""Reference Mamba mixer, calibration, and the quantized (W8A8) mixer (oracle side; test
infrastructure).  Plain numpy, sequential recurrence, dense Hadamard product.

Notation follows the paper: u block input, x the scan input (conv output), z the gate
branch, dt / B / C the selection outputs, A, D the SSM weights, y the scan output,
y^H = H_n y its Hadamard transform (Sections 3.1, 4.2, 4.3).

Weight layout (PyTorch [out, in] rows): W_in [2Di, Dm] rows x | z; conv_w [Di, W];
W_x [R+2N, Di] rows dt | B | C; W_dt [Di, R]; W_out [Dm, Di].
"""
from __future__ import annotations

import numpy as np

from .hadamard import hadamard_matrix
from .quantizer import absmax_scale, int_matmul, optimal_clip, percentile_max, quantize, requant_acc

F64 = np.float64
F32 = np.float32


# ----------------------------------------------------------------------------- elementwise
def silu(v):
    """SiLU(v) = v * sigmoid(v) = v / (1 + exp(-v)) (Section 3.1 gate, Section 4.3 conv)."""
    return v / (1.0 + np.exp(-v))


def softplus(v):
    """softplus(v) = log(1 + exp(v)), passed through unchanged above 20 (Section 3.1)."""
    v = np.asarray(v)
    return np.where(v > 20.0, v, np.log1p(np.exp(np.minimum(v, 20.0))))


# ----------------------------------------------------------------------------- operators
def causal_conv_fp(x_pre, conv_w, conv_b, history=None):
    """Depthwise causal convolution over time (Section 4.3, "Fused causal convolution"):
    out[b, t, d] = conv_b[d] + sum_j conv_w[d, j] * x_pre[b, t - (W-1) + j, d], taps before
    the sequence start come from ``history`` [B, W-1, Di] (zeros when None)."""
    Bt, L, Di = x_pre.shape
    W = conv_w.shape[1]
    hist = np.zeros((Bt, W - 1, Di), dtype=x_pre.dtype) if history is None else history
    ext = np.concatenate([hist, x_pre], axis=1)  # [B, W-1+L, Di]
    out = np.zeros((Bt, L, Di), dtype=np.result_type(x_pre.dtype, conv_w.dtype))
    for j in range(W):
        out = out + ext[:, j:j + L, :] * conv_w[:, j]
    return out + conv_b


def selective_scan(x, dt, A, Bm, Cm, D, z, h0=None):
    """Eq. 1 with selection, in fp64, one time step after the other:
        h_t = exp(dt_t A) h_{t-1} + dt_t B_t x_t,   y_t = C_t . h_t + D x_t,   g_t = y_t SiLU(z_t)
    (the paper's simplification B_dot ~= dt B).  x, dt, z [Bt, L, Di]; A [Di, N];
    Bm, Cm [Bt, L, N]; D [Di]; h0 [Bt, Di, N] or None.  Returns (g, y, h_L)."""
    x, dt, z = (np.asarray(v, dtype=F64) for v in (x, dt, z))
    A, Bm, Cm, D = (np.asarray(v, dtype=F64) for v in (A, Bm, Cm, D))
    Bt, L, Di = x.shape
    N = A.shape[1]
    h = np.zeros((Bt, Di, N), dtype=F64) if h0 is None else np.array(h0, dtype=F64)
    y = np.empty((Bt, L, Di), dtype=F64)
    for t in range(L):
        dA = np.exp(dt[:, t, :, None] * A[None, :, :])
        dBx = (dt[:, t, :] * x[:, t, :])[:, :, None] * Bm[:, t, None, :]
        h = dA * h + dBx
        y[:, t, :] = np.sum(h * Cm[:, t, None, :], axis=-1) + D * x[:, t, :]
    g = y * silu(z)
    return g, y, h


# ----------------------------------------------------------------------------- fp mixer
def fp_forward(w, u, h0=None, conv_history=None):
    """Unquantized Mamba mixer in fp64 (Section 3.1): in_proj -> causal conv + SiLU ->
    x_proj / dt_proj (+bias, softplus) -> selective scan -> gate -> out_proj.
    ``u`` [Bt, L, Dm].  Returns a dict of every intermediate."""
    u = np.asarray(u, dtype=F64)
    W_in, W_x, W_dt, W_out = (np.asarray(w[k], dtype=F64) for k in ("W_in", "W_x", "W_dt", "W_out"))
    Di = W_in.shape[0] // 2
    R = W_dt.shape[1]
    N = (W_x.shape[0] - R) // 2
    A = -np.exp(np.asarray(w["A_log"], dtype=F64))
    xz = u @ W_in.T
    x_pre, z = xz[..., :Di], xz[..., Di:]
    x = silu(causal_conv_fp(x_pre, np.asarray(w["conv_w"], dtype=F64),
                            np.asarray(w["conv_b"], dtype=F64), conv_history))
    dbc = x @ W_x.T
    dt_low, Bm, Cm = dbc[..., :R], dbc[..., R:R + N], dbc[..., R + N:]
    dt_raw = dt_low @ W_dt.T
    dt = softplus(dt_raw + np.asarray(w["dt_bias"], dtype=F64))
    g, y, h = selective_scan(x, dt, A, Bm, Cm, np.asarray(w["D"], dtype=F64), z, h0)
    out = g @ W_out.T
    return dict(u=u, x_pre=x_pre, z=z, x=x, dt_low=dt_low, B=Bm, C=Cm, dt_raw=dt_raw, dt=dt,
                y=y, g=g, out=out, h=h, A=A)


# ----------------------------------------------------------------------------- calibration
def calibrate(w, calib_u, x_percentile=99.999, x_clip="percentile"):
    """Static per-tensor scales and int8 weights (Section 5.1 "Quantization setup",
    Section 4.2): run the fp mixer on the calibration batch; every activation scale is
    absmax/127 except the scan input x, which takes the percentile maximum; the scale of
    y^H is collected after applying H_n to the gated scan output; W_out is replaced by
    W_out^H (each row transformed by the same H_n) before it is quantized.

    x_clip = "mse" replaces the percentile by the model-optimal clipping scalar
    (`quantizer.optimal_clip`), the enhanced variant Section 5.1 mentions; the paper does not say
    which tensors it clips, this reading applies it where the percentile was.

    Returns (qw, sc): int8 weights (+ fp32 conv_b, dt_bias) and a dict of fp32 scales
    and fp32 epilogue multipliers (products of scales evaluated in double, rounded once)."""
    t = fp_forward(w, calib_u)
    Dm = w["W_in"].shape[1]
    Di = w["W_in"].shape[0] // 2
    H = hadamard_matrix(Di).astype(F64)
    gH = t["g"] @ H.T  # y^H = H_n g for every token row
    W_outH = np.asarray(w["W_out"], dtype=F64) @ H.T  # row m: H_n W_out[m, :]
    A = t["A"]
    if x_clip == "percentile":
        x_clip_value = percentile_max(t["x"], x_percentile)
    elif x_clip == "mse":
        x_clip_value = optimal_clip(np.asarray(t["x"], dtype=F64).astype(F32))
    else:
        raise ValueError("x_clip must be 'percentile' or 'mse'")

    sc = {
        "s_u": absmax_scale(t["u"]), "s_xpre": absmax_scale(t["x_pre"]), "s_z": absmax_scale(t["z"]),
        "s_x": F32(x_clip_value / 127.0),
        "s_dtl": absmax_scale(t["dt_low"]), "s_B": absmax_scale(t["B"]), "s_C": absmax_scale(t["C"]),
        "s_dt": absmax_scale(t["dt_raw"]), "s_y": absmax_scale(gH),
        "s_Win": absmax_scale(w["W_in"]), "s_cw": absmax_scale(w["conv_w"]),
        "s_Wx": absmax_scale(w["W_x"]), "s_Wdt": absmax_scale(w["W_dt"]),
        "s_A": absmax_scale(A), "s_D": absmax_scale(w["D"]), "s_WoutH": absmax_scale(W_outH),
    }
    if sc["s_x"] <= 0:
        sc["s_x"] = F32(1.0)
    d = {k: float(v) for k, v in sc.items()}
    sc.update({
        "inv_s_u": F32(1.0 / d["s_u"]),
        "m_in_x": F32(d["s_u"] * d["s_Win"] / d["s_xpre"]),
        "m_in_z": F32(d["s_u"] * d["s_Win"] / d["s_z"]),
        "m_conv": F32(d["s_cw"] * d["s_xpre"]),
        "inv_s_x": F32(1.0 / d["s_x"]),
        "m_x_dt": F32(d["s_x"] * d["s_Wx"] / d["s_dtl"]),
        "m_x_B": F32(d["s_x"] * d["s_Wx"] / d["s_B"]),
        "m_x_C": F32(d["s_x"] * d["s_Wx"] / d["s_C"]),
        "m_dt": F32(d["s_dtl"] * d["s_Wdt"] / d["s_dt"]),
        "inv_s_y": F32(1.0 / d["s_y"]),
        "m_out": F32(d["s_y"] * d["s_WoutH"] / Di),
    })

    def qwt(X, s):
        return quantize(np.asarray(X, dtype=F64).astype(F32), F32(1.0 / float(s)))

    qw = {
        "W_in": qwt(w["W_in"], sc["s_Win"]), "conv_w": qwt(w["conv_w"], sc["s_cw"]),
        "W_x": qwt(w["W_x"], sc["s_Wx"]), "W_dt": qwt(w["W_dt"], sc["s_Wdt"]),
        "A": qwt(A, sc["s_A"]), "D": qwt(w["D"], sc["s_D"]),
        "W_outH": qwt(W_outH, sc["s_WoutH"]),
        "conv_b": np.asarray(w["conv_b"], dtype=F32), "dt_bias": np.asarray(w["dt_bias"], dtype=F32),
    }
    assert qw["W_outH"].shape == (Dm, Di)
    return qw, sc


# ----------------------------------------------------------------------------- quantized mixer
def _dims(qw):
    Di = qw["W_in"].shape[0] // 2
    R = qw["W_dt"].shape[1]
    N = (qw["W_x"].shape[0] - R) // 2
    return Di, R, N


def _silu32(v):
    v = np.asarray(v, dtype=F32)
    return (v / (F32(1.0) + np.exp(-v))).astype(F32)


def q_scan(x_q, dt_q, z_q, B_q, C_q, A_q, D_q, dt_bias, sc, h0=None, x_values=None):
    """Quantized selective SSM of Section 4.2: int8 x, dt, B, C, z and int8 weights A, D go in
    with their static scales and are dequantized inside; dt gets its fp32 bias and the
    softplus after dequantization; the output is rounded to half precision.
    Shapes: x_q, dt_q, z_q [Bt, L, Dsub]; B_q, C_q [Bt, L, N]; A_q [Dsub, N]; D_q, dt_bias
    [Dsub] (any subset of channels works: channels do not interact).
    ``x_values`` (a half-precision x given directly) replaces s_x * x_q: the comparison
    variant of Appendix H feeds the scan an x that went through a transform pair instead.
    Returns (g fp64, g16 fp16, h_L fp32)."""
    f = lambda k: float(sc[k])  # noqa: E731
    x = f("s_x") * np.asarray(x_q).astype(F64) if x_values is None else np.asarray(x_values).astype(F64)
    dt = softplus(f("s_dt") * np.asarray(dt_q).astype(F64) + np.asarray(dt_bias).astype(F64))
    A = f("s_A") * np.asarray(A_q).astype(F64)
    Bm = f("s_B") * np.asarray(B_q).astype(F64)
    Cm = f("s_C") * np.asarray(C_q).astype(F64)
    D = f("s_D") * np.asarray(D_q).astype(F64)
    z = f("s_z") * np.asarray(z_q).astype(F64)
    g, _, h = selective_scan(x, dt, A, Bm, Cm, D, z, h0)
    return g, g.astype(np.float16), h.astype(F32)


def q_hadamard_quant(g16, sc):
    """Eq. 3: y^H = H_n g (dense fp64 product over the fp16 rows), then
    clamp(rne(fp32(y^H) * fp32(1/s_y))).  g16 [..., n].  Returns (y^H fp64, int8)."""
    n = g16.shape[-1]
    H = hadamard_matrix(n).astype(F64)
    gH = np.asarray(g16).astype(F64) @ H.T
    return gH, quantize(gH.astype(F32), sc["inv_s_y"])


def q_out_proj(gH_q, W_outH_q, sc):
    """Output projection with the folded weight (Section 4.2 fold identity; Section 4.3: half
    precision out): fp16(fp32(acc) * m_out), m_out = s_y s_WoutH / n."""
    shp = gH_q.shape
    acc = int_matmul(gH_q.reshape(-1, shp[-1]), W_outH_q).reshape(*shp[:-1], -1)
    return acc, (acc.astype(F32) * F32(sc["m_out"])).astype(np.float16)


def conv_prefill_silu(xpre_q, conv_w_q, conv_b, sc):
    """SiLU(Conv(x_in_q, W_q, s)), s = s_w s_xin, from an empty history (Section 4.3 before the
    output quantizer): integer taps, then fp32 (acc * m_conv + bias), SiLU in fp32.
    xpre_q [Bt, L, Dsub]; conv_w_q [Dsub, W]; conv_b [Dsub]."""
    Dsub = xpre_q.shape[-1]
    conv_acc = causal_conv_fp(np.asarray(xpre_q).astype(np.int32), np.asarray(conv_w_q).astype(np.int32),
                              np.zeros(Dsub, dtype=np.int32))
    v = conv_acc.astype(F32) * F32(sc["m_conv"]) + np.asarray(conv_b).astype(F32)
    return _silu32(v)


def q_conv_prefill(xpre_q, conv_w_q, conv_b, sc):
    """Section 4.3: x_out = (1/s_out) SiLU(Conv(x_in_q, W_q, s)): `conv_prefill_silu`, then the
    quantizer with the percentile scale of x."""
    return quantize(conv_prefill_silu(xpre_q, conv_w_q, conv_b, sc), sc["inv_s_x"])


def conv_step_silu(xpre_q_new, conv_state, conv_w_q, conv_b, sc):
    """Decode form before the output quantizer: fp32 conv over [conv_state (W-1, fp16),
    s_xpre * x_pre_q] with weights s_cw * w_q, accumulated oldest tap first on top of the
    bias, SiLU in fp32; then the window shifts.
    xpre_q_new [Bt, Dsub]; conv_state [Bt, Dsub, W-1].  Returns (x fp32 [Bt, Dsub], new state)."""
    new = (F32(sc["s_xpre"]) * np.asarray(xpre_q_new).astype(F32)).astype(F32)
    win = np.concatenate([np.asarray(conv_state).astype(F32), new[:, :, None]], axis=2)
    wdq = (F32(sc["s_cw"]) * np.asarray(conv_w_q).astype(F32)).astype(F32)
    v = np.asarray(conv_b).astype(F32)[None, :].repeat(win.shape[0], axis=0)
    for j in range(wdq.shape[1]):
        v = (v + (wdq[None, :, j] * win[:, :, j]).astype(F32)).astype(F32)
    return _silu32(v), win[:, :, 1:].astype(np.float16)


def q_conv_step(xpre_q_new, conv_state, conv_w_q, conv_b, sc):
    """`conv_step_silu`, then the quantizer with the percentile scale of x.
    Returns (x_q [Bt, Dsub], new state)."""
    x, new_state = conv_step_silu(xpre_q_new, conv_state, conv_w_q, conv_b, sc)
    return quantize(x, sc["inv_s_x"]), new_state


def _scan_and_tail(qw, sc, t, x_q, z_q, dt_q, B_q, C_q, h0):
    """Steps shared by prefill and decode after the projections: scan + gate, Hadamard +
    quantize, output projection."""
    g, g16, h = q_scan(x_q, dt_q, z_q, B_q, C_q, qw["A"], qw["D"], qw["dt_bias"], sc, h0)
    gH, gH_q = q_hadamard_quant(g16, sc)
    acc_out, out = q_out_proj(gH_q, qw["W_outH"], sc)
    t.update(g=g, g16=g16, gH=gH, gH_q=gH_q, acc_out=acc_out, out=out, h=h)
    return t


def _projections(qw, sc, x_q):
    """x_proj and dt_proj on int8 (Section 3.1 selection; Section 4.2: their weights are
    8-bit): accumulator columns [0,R) -> dt_low, [R,R+N) -> B, [R+N,R+2N) -> C, each with
    its own output scale; dt is requantized before the bias and the softplus, which the
    scan applies after dequantizing."""
    Di, R, N = _dims(qw)
    Bt, L, _ = x_q.shape
    acc_x = int_matmul(x_q.reshape(Bt * L, Di), qw["W_x"]).reshape(Bt, L, R + 2 * N)
    dtl_q = requant_acc(acc_x[..., :R], sc["m_x_dt"])
    B_q = requant_acc(acc_x[..., R:R + N], sc["m_x_B"])
    C_q = requant_acc(acc_x[..., R + N:], sc["m_x_C"])
    acc_dt = int_matmul(dtl_q.reshape(Bt * L, R), qw["W_dt"]).reshape(Bt, L, Di)
    dt_q = requant_acc(acc_dt, sc["m_dt"])
    return dict(acc_x=acc_x, dtl_q=dtl_q, B_q=B_q, C_q=C_q, acc_dt=acc_dt, dt_q=dt_q)


def _in_proj(qw, sc, u=None, u_q=None):
    Di, R, N = _dims(qw)
    if u_q is None:
        u_q = quantize(np.asarray(u).astype(F32), sc["inv_s_u"])
    Bt, L, Dm = u_q.shape
    acc_in = int_matmul(u_q.reshape(Bt * L, Dm), qw["W_in"]).reshape(Bt, L, 2 * Di)
    xpre_q = requant_acc(acc_in[..., :Di], sc["m_in_x"])
    z_q = requant_acc(acc_in[..., Di:], sc["m_in_z"])
    return dict(u_q=u_q, acc_in=acc_in, xpre_q=xpre_q, z_q=z_q)


def q_prefill(qw, sc, u=None, h0=None, u_q=None):
    """Quantized mixer over a whole sequence from an empty conv history.
    ``u`` fp16 [Bt, L, Dm] (or ``u_q`` int8, already quantized with s_u).  Returns every
    intermediate; ``out`` fp16 [Bt, L, Dm], ``h`` fp32 [Bt, Di, N], ``conv_state`` fp16
    [Bt, Di, W-1] (the last W-1 dequantized conv inputs, oldest first)."""
    Di, R, N = _dims(qw)
    t = _in_proj(qw, sc, u, u_q)
    xpre_q, z_q = t["xpre_q"], t["z_q"]
    Bt, L, _ = xpre_q.shape
    W = qw["conv_w"].shape[1]
    x_q = q_conv_prefill(xpre_q, qw["conv_w"], qw["conv_b"], sc)
    t.update(x_q=x_q)
    t.update(_projections(qw, sc, x_q))
    _scan_and_tail(qw, sc, t, x_q, z_q, t["dt_q"], t["B_q"], t["C_q"], h0)
    hist = np.zeros((Bt, W - 1, Di), dtype=F32)
    take = min(L, W - 1)
    hist[:, W - 1 - take:, :] = F32(sc["s_xpre"]) * xpre_q[:, L - take:, :].astype(F32)
    t["conv_state"] = np.ascontiguousarray(hist.transpose(0, 2, 1)).astype(np.float16)
    return t


def q_decode(qw, sc, u, ssm_state, conv_state, u_q=None):
    """One generation step.  ``u`` fp16 [Bt, Dm]; ``ssm_state`` fp32 [Bt, Di, N];
    ``conv_state`` fp16 [Bt, Di, W-1] holding dequantized conv inputs, oldest first.
    The conv runs in fp32 over [state, s_xpre * x_pre_q] with the dequantized weights;
    the window then shifts by one.  Returns the intermediates plus the new states."""
    Di, R, N = _dims(qw)
    t = _in_proj(qw, sc, None if u is None else np.asarray(u)[:, None, :],
                 None if u_q is None else np.asarray(u_q)[:, None, :])
    xpre_q, z_q = t["xpre_q"], t["z_q"]  # [Bt, 1, Di]
    x_q2, new_state = q_conv_step(xpre_q[:, 0, :], conv_state, qw["conv_w"], qw["conv_b"], sc)
    x_q = x_q2[:, None, :]
    t.update(x_q=x_q)
    t.update(_projections(qw, sc, x_q))
    _scan_and_tail(qw, sc, t, x_q, z_q, t["dt_q"], t["B_q"], t["C_q"], ssm_state)
    t["conv_state"] = new_state
    return t


# ----------------------------------------------------------------------------- block glue
def add_rmsnorm_quant(x_out, x_res, weight, inv_s, eps=1e-5):
    """Section 4.3 "Fused RMSNorm": (q(RMSNorm(x_out + x_res)), x_out + x_res).
    The sum is formed in fp32 and stored as fp16; the norm is taken over that stored
    residual (fp64 mean of squares), scaled by the fp16 weight, and quantized with the
    next block's input scale."""
    s = (np.asarray(x_out).astype(F32) + np.asarray(x_res).astype(F32)).astype(np.float16)
    r = s.astype(F64)
    ms = np.mean(r * r, axis=-1, keepdims=True)
    y = r / np.sqrt(ms + eps) * np.asarray(weight).astype(F64)
    return quantize(y.astype(F32), inv_s), s
