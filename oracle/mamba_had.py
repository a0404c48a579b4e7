"""The comparison variant of Appendix H ("Mamba-Had": the rotation recipe for Transformers moved onto
the Mamba block) on the scan-input path (oracle side; test infrastructure).

Appendix H gives the sequence for the scan input: causal conv -> forward Hadamard & quantize ->
backward Hadamard -> selective scan, with the Hadamard matrices folded into the linear layers
(figure caption).  The figure itself is not available, so the wiring below is a reading:

  x16   = fp16(SiLU(conv(x_pre_q)))                           conv output, not quantized
  xH_q  = q(H_n x16, s_xH),  s_xH = max|H_n x| / 127          forward transform + quantize
  x_proj consumes xH_q with W_xH = q(rows of W_x transformed by the same H_n) and 1/n in the
          multiplier: (H w) . (H x) = n (w . x)                the fold into the linear layer
  x_hat = fp16((s_xH / n) H_n^T xH_q)                         backward transform
  the scan takes x_hat in half precision where Quamba's takes s_x * x_q

Everything else (in_proj, dt_proj, the int8 B, C, dt, z of the scan, the output Hadamard and
out_proj) is the Quamba path unchanged.  The paper's transposes between the conv and scan layouts
are artefacts of the kernels it reused and have no counterpart here.

Pins (tests/test_oracle_mamba_had.py): the transform pair returns its input exactly (which fixes H
versus H^T for the non-symmetric Paley factors), the folded x_proj weight reproduces W_x x, the
reconstruction error of x_hat is the rounding noise the rotated grid implies (bound and RMS), the
variant tracks the unquantized mixer on par with Quamba, and a decode step continues a prefill.
parity unpinned: the end-to-end numbers (the paper prints no worked example of this variant).
"""
from __future__ import annotations

import numpy as np

from .hadamard import hadamard_matrix
from .mixer import (_dims, _in_proj, calibrate, conv_prefill_silu, conv_step_silu, fp_forward, q_hadamard_quant,
                    q_out_proj, q_scan)
from .quantizer import absmax_scale, int_matmul, quantize, requant_acc

F32, F64 = np.float32, np.float64


def calibrate_hadx(w, calib_u, x_percentile=99.999):
    """Quamba's calibration plus what the variant needs: the scale of H_n x over the calibration
    batch (absmax; the rotation is there to make the maximum harmless), the rotated and quantized
    x_proj weight, and the multipliers.  Returns (qw, sc, hx)."""
    qw, sc = calibrate(w, calib_u, x_percentile)
    t = fp_forward(w, calib_u)
    Di = w["W_in"].shape[0] // 2
    H = hadamard_matrix(Di).astype(F64)
    xH = t["x"] @ H.T                                   # H_n x for every token row
    W_xH = np.asarray(w["W_x"], dtype=F64) @ H.T        # row r: H_n W_x[r, :]
    s_xH, s_WxH = absmax_scale(xH), absmax_scale(W_xH)
    d = {k: float(v) for k, v in sc.items()}
    a, b = float(s_xH), float(s_WxH)
    hx = {
        "W_xH": quantize(W_xH.astype(F32), F32(1.0 / b)), "W_xH_fp": W_xH,
        "s_xH": s_xH, "s_WxH": s_WxH, "inv_s_xH": F32(1.0 / a),
        "m_xh_dt": F32(a * b / (Di * d["s_dtl"])), "m_xh_B": F32(a * b / (Di * d["s_B"])),
        "m_xh_C": F32(a * b / (Di * d["s_C"])), "xhat_scale": F32(a / Di),
    }
    return qw, sc, hx


def hadamard_inverse_dequant(xH_q, scale):
    """x_hat = fp16(fp32(scale) * (H_n^T xH_q)); the integer sums are exact."""
    n = xH_q.shape[-1]
    H = hadamard_matrix(n).astype(F64)
    back = np.asarray(xH_q).astype(F64) @ H             # row form of H^T v
    return (back.astype(F32) * F32(scale)).astype(np.float16)


def _x_path(qw, sc, hx, x32, t):
    """From the conv output (fp32) to the projections' int8 outputs and the scan's x_hat."""
    Di, R, N = _dims(qw)
    x16 = np.asarray(x32, dtype=F32).astype(np.float16)
    lead = x16.shape[:-1]
    H = hadamard_matrix(Di).astype(F64)
    xH = x16.astype(F64) @ H.T
    xH_q = quantize(xH.astype(F32), hx["inv_s_xH"])
    acc_x = int_matmul(xH_q.reshape(-1, Di), hx["W_xH"]).reshape(*lead, R + 2 * N)
    dtl_q = requant_acc(acc_x[..., :R], hx["m_xh_dt"])
    B_q = requant_acc(acc_x[..., R:R + N], hx["m_xh_B"])
    C_q = requant_acc(acc_x[..., R + N:], hx["m_xh_C"])
    acc_dt = int_matmul(dtl_q.reshape(-1, R), qw["W_dt"]).reshape(*lead, Di)
    dt_q = requant_acc(acc_dt, sc["m_dt"])
    xhat16 = hadamard_inverse_dequant(xH_q, hx["xhat_scale"])
    t.update(x16=x16, xH=xH, xH_q=xH_q, acc_x=acc_x, dtl_q=dtl_q, B_q=B_q, C_q=C_q, acc_dt=acc_dt, dt_q=dt_q,
             xhat16=xhat16)
    return t


def _tail(qw, sc, t, z_q, h0):
    """Scan on x_hat + gate, output Hadamard + quantize, out_proj: the Quamba steps."""
    g, g16, h = q_scan(None, t["dt_q"], z_q, t["B_q"], t["C_q"], qw["A"], qw["D"], qw["dt_bias"], sc, h0,
                       x_values=t["xhat16"])
    gH, gH_q = q_hadamard_quant(g16, sc)
    acc_out, out = q_out_proj(gH_q, qw["W_outH"], sc)
    t.update(g=g, g16=g16, gH=gH, gH_q=gH_q, acc_out=acc_out, out=out, h=h)
    return t


def q_prefill_hadx(qw, sc, hx, u=None, h0=None, u_q=None):
    """The variant over whole sequences from an empty conv history; same arguments and results as
    `q_prefill`, plus hx and the intermediates x16, xH_q, xhat16."""
    Di, R, N = _dims(qw)
    t = _in_proj(qw, sc, u, u_q)
    xpre_q, z_q = t["xpre_q"], t["z_q"]
    Bt, L, _ = xpre_q.shape
    W = qw["conv_w"].shape[1]
    _x_path(qw, sc, hx, conv_prefill_silu(xpre_q, qw["conv_w"], qw["conv_b"], sc), t)
    _tail(qw, sc, t, z_q, h0)
    hist = np.zeros((Bt, W - 1, Di), dtype=F32)
    take = min(L, W - 1)
    hist[:, W - 1 - take:, :] = F32(sc["s_xpre"]) * xpre_q[:, L - take:, :].astype(F32)
    t["conv_state"] = np.ascontiguousarray(hist.transpose(0, 2, 1)).astype(np.float16)
    return t


def q_decode_hadx(qw, sc, hx, u, ssm_state, conv_state, u_q=None):
    """One generation step of the variant; arguments and results as `q_decode`, plus hx."""
    t = _in_proj(qw, sc, None if u is None else np.asarray(u)[:, None, :],
                 None if u_q is None else np.asarray(u_q)[:, None, :])
    xpre_q, z_q = t["xpre_q"], t["z_q"]
    x32, new_state = conv_step_silu(xpre_q[:, 0, :], conv_state, qw["conv_w"], qw["conv_b"], sc)
    _x_path(qw, sc, hx, x32[:, None, :], t)
    _tail(qw, sc, t, z_q, ssm_state)
    t["conv_state"] = new_state
    return t
