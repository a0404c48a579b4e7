"""Dynamic 8-bit quantization of the scan input x (Appendix K, row "Dynamic / MinMax Sym."; oracle
side, test infrastructure).

Appendix K: the scale of x is not calibrated but taken from the values at hand, which closes most of
the accuracy gap at the price of recomputing the scale on every call.  The paper gives no formulas;
the reading (one scale per call, over everything the call processes):

  x16  = fp16(SiLU(conv(x_pre_q)))                       the conv output, kept in half precision
  s    = fp32(max|x16|) / fp32(127)   (1 if the maximum is 0)          one fp32 division
  x_q  = clamp(rne(fp32(x16) * fp32(1 / s)), -128, 127)                1 / s: one fp32 division
  x_proj: int32 sums over x_q, outputs clamp(rne(fp32(acc) * m)) with m = fp32(fp32(s * s_Wx) / s_out)
  scan:  x = s * x_q

Every fp32 operation above is written in the order the device performs it, so both sides reach the
same scale bit for bit and the same codes.  Everything else is the Quamba path; the calibrated s_x
is simply not used.  Pins (tests/test_oracle_x_dynamic.py): the scale is the one of Eq. 2 on the
call's own values and the largest value lands on +-127, the error of the codes never exceeds that of
a static scale taken from other data, a call that is scaled by a constant gives the same codes,
the variant tracks the unquantized mixer at least as well as the static absmax rule on data whose
range differs from the calibration's, decode continues prefill.
parity unpinned: the end-to-end numbers (the paper prints accuracy on its datasets only).
"""
from __future__ import annotations

import numpy as np

from .mixer import (_dims, _in_proj, conv_prefill_silu, conv_step_silu, q_hadamard_quant, q_out_proj, q_scan)
from .quantizer import QMAX, int_matmul, quantize, requant_acc

F32, F64 = np.float32, np.float64


def dynamic_scale(x16):
    """(s, 1/s, as fp32) from the half-precision values of one call."""
    mx = F32(np.max(np.abs(np.asarray(x16, dtype=np.float16).astype(F32)))) if np.size(x16) else F32(0)
    s = F32(mx / F32(QMAX)) if mx > 0 else F32(1.0)
    return s, F32(F32(1.0) / s)


def dynamic_multipliers(s, sc):
    """The three output multipliers of x_proj for the call's scale: fp32(fp32(s * s_Wx) / s_out)."""
    p = F32(F32(s) * F32(sc["s_Wx"]))
    return F32(p / F32(sc["s_dtl"])), F32(p / F32(sc["s_B"])), F32(p / F32(sc["s_C"]))


def _x_path(qw, sc, x32, t):
    Di, R, N = _dims(qw)
    x16 = np.asarray(x32, dtype=F32).astype(np.float16)
    s, inv_s = dynamic_scale(x16)
    x_q = quantize(x16.astype(F32), inv_s)
    m_dt, m_B, m_C = dynamic_multipliers(s, sc)
    lead = x_q.shape[:-1]
    acc_x = int_matmul(x_q.reshape(-1, Di), qw["W_x"]).reshape(*lead, R + 2 * N)
    dtl_q = requant_acc(acc_x[..., :R], m_dt)
    B_q = requant_acc(acc_x[..., R:R + N], m_B)
    C_q = requant_acc(acc_x[..., R + N:], m_C)
    acc_dt = int_matmul(dtl_q.reshape(-1, R), qw["W_dt"]).reshape(*lead, Di)
    dt_q = requant_acc(acc_dt, sc["m_dt"])
    x_deq = (s * x_q.astype(F32)).astype(F32)
    t.update(x16=x16, s_x_dyn=s, x_q=x_q, acc_x=acc_x, dtl_q=dtl_q, B_q=B_q, C_q=C_q, acc_dt=acc_dt, dt_q=dt_q, x_deq=x_deq)
    return t


def _tail(qw, sc, t, z_q, h0):
    g, g16, h = q_scan(None, t["dt_q"], z_q, t["B_q"], t["C_q"], qw["A"], qw["D"], qw["dt_bias"], sc, h0,
                       x_values=t["x_deq"])
    gH, gH_q = q_hadamard_quant(g16, sc)
    acc_out, out = q_out_proj(gH_q, qw["W_outH"], sc)
    t.update(g=g, g16=g16, gH=gH, gH_q=gH_q, acc_out=acc_out, out=out, h=h)
    return t


def q_prefill_xdyn(qw, sc, u=None, h0=None, u_q=None):
    """The quantized mixer with a per-call scale of x, whole sequences from an empty conv history;
    arguments and results as `q_prefill` (qw, sc from `calibrate`)."""
    Di, R, N = _dims(qw)
    t = _in_proj(qw, sc, u, u_q)
    xpre_q, z_q = t["xpre_q"], t["z_q"]
    Bt, L, _ = xpre_q.shape
    W = qw["conv_w"].shape[1]
    _x_path(qw, sc, conv_prefill_silu(xpre_q, qw["conv_w"], qw["conv_b"], sc), t)
    _tail(qw, sc, t, z_q, h0)
    hist = np.zeros((Bt, W - 1, Di), dtype=F32)
    take = min(L, W - 1)
    hist[:, W - 1 - take:, :] = F32(sc["s_xpre"]) * xpre_q[:, L - take:, :].astype(F32)
    t["conv_state"] = np.ascontiguousarray(hist.transpose(0, 2, 1)).astype(np.float16)
    return t


def q_decode_xdyn(qw, sc, u, ssm_state, conv_state, u_q=None):
    """One generation step with the scale of x taken from this step's values (all sequences of the
    step together); arguments and results as `q_decode`."""
    t = _in_proj(qw, sc, None if u is None else np.asarray(u)[:, None, :],
                 None if u_q is None else np.asarray(u_q)[:, None, :])
    xpre_q, z_q = t["xpre_q"], t["z_q"]
    x32, new_state = conv_step_silu(xpre_q[:, 0, :], conv_state, qw["conv_w"], qw["conv_b"], sc)
    _x_path(qw, sc, x32[:, None, :], t)
    _tail(qw, sc, t, z_q, ssm_state)
    t["conv_state"] = new_state
    return t
