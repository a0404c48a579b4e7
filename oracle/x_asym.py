"""Asymmetric 8-bit quantizer with percentile clipping for the scan input x (Appendix K, row
"MinMax Asym. Per."; oracle side, test infrastructure).

Appendix K observes that x (the output of SiLU) is far from symmetric and that an asymmetric grid
uses the 8 bits better, at the price of extra work in the operators that read x.  The paper gives
no formulas, so this is a reading (uniform affine quantizer, zero point in the code domain):

  lo = min(min x, 0),  hi = max^p(|x|) (the percentile maximum Quamba uses),  s = (hi - lo) / 255
  zp = clamp(rne(-128 - lo / s), -128, 127)
  x_q = clamp(rne(fp32(fp32(x) * fp32(1/s)) + zp), -128, 127)          (conv epilogue)
  x   = s * (x_q - zp)                                                  (inside the scan)
  x_proj:  sum_k W_q[n, k] (x_q[k] - zp) = acc[n] - zp * rowsum(W_q[n, :])   (an int32 term per
           output column, added before the requantization; multiplier s * s_Wx / s_out)

Everything else is the Quamba path.  Pins (tests/test_oracle_x_asym.py): round trip within s / 2 and
both ends of the range reached, the column correction against a brute-force product of the shifted
codes, the step being (127 / 255) (1 - lo / hi) times the symmetric one and the error of the x codes
shrinking with it, the error against the unquantized mixer not above Quamba's, decode continuing
prefill.
parity unpinned: the end-to-end numbers (the paper prints accuracy on its datasets only).
"""
from __future__ import annotations

import numpy as np

from .mixer import (_dims, _in_proj, calibrate, conv_prefill_silu, conv_step_silu, fp_forward, q_hadamard_quant,
                    q_out_proj, q_scan)
from .quantizer import QMAX, QMIN, int_matmul, percentile_max, requant_acc, rne

F32, F64 = np.float32, np.float64


def quantize_asym(v, inv_s, zp) -> np.ndarray:
    """clamp(rne(fp32(fp32(v) * fp32(1/s)) + zp), -128, 127): one fp32 multiply, one fp32 add, one rounding."""
    t = (np.asarray(v, dtype=F32) * F32(inv_s)).astype(F32) + F32(zp)
    return np.clip(rne(t.astype(F32)), QMIN, QMAX).astype(np.int8)


def calibrate_xasym(w, calib_u, x_percentile=99.999):
    """Quamba's calibration plus the asymmetric grid of x.  Returns (qw, sc, xa)."""
    qw, sc = calibrate(w, calib_u, x_percentile)
    x = np.asarray(fp_forward(w, calib_u)["x"], dtype=F64)
    lo = min(float(x.min()), 0.0)
    hi = percentile_max(x, x_percentile)
    span = hi - lo
    s = F32(span / 255.0) if span > 0.0 else F32(1.0)
    zp = int(np.clip(np.rint(-128.0 - lo / float(s)), QMIN, QMAX))
    d = {k: float(v) for k, v in sc.items()}
    rowsum = qw["W_x"].astype(np.int64).sum(axis=1)
    xa = {
        "s_x": s, "inv_s_x": F32(1.0 / float(s)), "zero_point": zp,
        "m_x_dt": F32(float(s) * d["s_Wx"] / d["s_dtl"]), "m_x_B": F32(float(s) * d["s_Wx"] / d["s_B"]),
        "m_x_C": F32(float(s) * d["s_Wx"] / d["s_C"]),
        "col_bias": (-zp * rowsum).astype(np.int32),
    }
    return qw, sc, xa


def _x_path(qw, sc, xa, x32, t):
    Di, R, N = _dims(qw)
    x_q = quantize_asym(x32, xa["inv_s_x"], xa["zero_point"])
    lead = x_q.shape[:-1]
    acc_x = int_matmul(x_q.reshape(-1, Di), qw["W_x"]).reshape(*lead, R + 2 * N)
    acc_c = (acc_x.astype(np.int64) + xa["col_bias"].astype(np.int64)).astype(np.int32)
    dtl_q = requant_acc(acc_c[..., :R], xa["m_x_dt"])
    B_q = requant_acc(acc_c[..., R:R + N], xa["m_x_B"])
    C_q = requant_acc(acc_c[..., R + N:], xa["m_x_C"])
    acc_dt = int_matmul(dtl_q.reshape(-1, R), qw["W_dt"]).reshape(*lead, Di)
    dt_q = requant_acc(acc_dt, sc["m_dt"])
    x_deq = (F32(xa["s_x"]) * (x_q.astype(F32) - F32(xa["zero_point"]))).astype(F32)
    t.update(x_q=x_q, acc_x=acc_x, dtl_q=dtl_q, B_q=B_q, C_q=C_q, acc_dt=acc_dt, dt_q=dt_q, x_deq=x_deq)
    return t


def _tail(qw, sc, t, z_q, h0):
    g, g16, h = q_scan(None, t["dt_q"], z_q, t["B_q"], t["C_q"], qw["A"], qw["D"], qw["dt_bias"], sc, h0,
                       x_values=t["x_deq"])
    gH, gH_q = q_hadamard_quant(g16, sc)
    acc_out, out = q_out_proj(gH_q, qw["W_outH"], sc)
    t.update(g=g, g16=g16, gH=gH, gH_q=gH_q, acc_out=acc_out, out=out, h=h)
    return t


def q_prefill_xasym(qw, sc, xa, u=None, h0=None, u_q=None):
    """The quantized mixer with the asymmetric x grid, whole sequences from an empty conv history;
    arguments and results as `q_prefill`, plus xa."""
    Di, R, N = _dims(qw)
    t = _in_proj(qw, sc, u, u_q)
    xpre_q, z_q = t["xpre_q"], t["z_q"]
    Bt, L, _ = xpre_q.shape
    W = qw["conv_w"].shape[1]
    _x_path(qw, sc, xa, conv_prefill_silu(xpre_q, qw["conv_w"], qw["conv_b"], sc), t)
    _tail(qw, sc, t, z_q, h0)
    hist = np.zeros((Bt, W - 1, Di), dtype=F32)
    take = min(L, W - 1)
    hist[:, W - 1 - take:, :] = F32(sc["s_xpre"]) * xpre_q[:, L - take:, :].astype(F32)
    t["conv_state"] = np.ascontiguousarray(hist.transpose(0, 2, 1)).astype(np.float16)
    return t


def q_decode_xasym(qw, sc, xa, u, ssm_state, conv_state, u_q=None):
    """One generation step with the asymmetric x grid; arguments and results as `q_decode`, plus xa."""
    t = _in_proj(qw, sc, None if u is None else np.asarray(u)[:, None, :],
                 None if u_q is None else np.asarray(u_q)[:, None, :])
    xpre_q, z_q = t["xpre_q"], t["z_q"]
    x32, new_state = conv_step_silu(xpre_q[:, 0, :], conv_state, qw["conv_w"], qw["conv_b"], sc)
    _x_path(qw, sc, xa, x32[:, None, :], t)
    _tail(qw, sc, t, z_q, ssm_state)
    t["conv_state"] = new_state
    return t
