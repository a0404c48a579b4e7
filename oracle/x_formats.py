"""Non-uniform 8-bit formats for the scan input x (Appendix K: row "MinMax Sym. Log2" and the
paragraph on low-bit floating point, E4M3; oracle side, test infrastructure).

Appendix K reports a log2 quantizer (every value goes to the nearest power of two) as slightly
better than Quamba's percentile grid but without a matrix-multiply form on the frameworks it used,
and names FP8 (E5M2 / E4M3) as something to explore.  It gives no formulas; the readings:

  log2   scale s = max|x| over the calibration batch (the row says MinMax), t = fp32(|x|) * fp32(1/s),
         written t = f 2^E with 1 <= f < 2;  k = E + (f >= fp32(sqrt 2))  (nearest power of two in the
         log domain: the midpoint between 2^E and 2^(E+1) is 2^(E+1/2));  e = clamp(-k, 0, .);
         values below 2^-126.5 (e > 126) and zero take the zero code.  Code byte: bit 7 = sign,
         bits 0..6 = e, 127 = zero.  x_hat = sign * s * 2^-e.
  e4m3   the OCP 8-bit float: 1 sign, 4 exponent bits (bias 7), 3 mantissa bits, subnormals
         m 2^-9, largest finite value 448 (0x7e), no infinities, 0x7f / 0xff not a number (never
         produced).  scale s = max^p(|x|) / 448 with Quamba's percentile; t = fp32(x) * fp32(1/s),
         rounded to the nearest representable value (ties to the even mantissa), saturating at
         +-448.  x_hat = s * value(code).

Both feed the scan (x = fp32(s) * value) and x_proj.  x_proj has a matrix form with exact operands:
the decoded values (dyadic, at most 4 significant bits) and the int8 weight codes are all
representable in bfloat16, so  acc[n] = sum_k W_q[n, k] value_k  is an ordinary real dot product
(fp64 here; a bf16 matrix unit with fp32 accumulation on the device), and the int8 outputs are
clamp(rne(fp32(acc) * m)), m = s_x s_Wx / s_out.  Everything else is the Quamba path.

Pins (tests/test_oracle_x_formats.py): the E4M3 table against the format's defining numbers, the
encoder against a brute-force nearest-value search over that table (ties, saturation, subnormals),
round trips of every code, the error bounds of both formats (2^-4 relative for normal E4M3 values,
a factor sqrt 2 for log2), the log2 rounding against a search in the log domain, x_proj against
exact rational arithmetic, the variants against the unquantized mixer and against Quamba on inputs
with outliers, decode continuing prefill.
parity unpinned: the end-to-end numbers (the paper prints accuracy on its datasets only).
"""
from __future__ import annotations

import numpy as np

from .mixer import (_dims, _in_proj, calibrate, conv_prefill_silu, conv_step_silu, fp_forward, q_hadamard_quant,
                    q_out_proj, q_scan)
from .quantizer import QMAX, QMIN, int_matmul, percentile_max, requant_acc, rne

F32, F64 = np.float32, np.float64
E4M3_MAX = 448.0
LOG2_ZERO = 127          # exponent field of the zero code
SQRT2_F32 = F32(1.4142135623730951)

FORMATS = ("e4m3", "log2")


# ------------------------------------------------------------------------------------ E4M3
def decode_e4m3(code) -> np.ndarray:
    """Value of each code byte (float64); the two not-a-number codes give nan."""
    c = np.asarray(code).astype(np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    ex = (c >> 3) & 0xF
    m = c & 0x7
    v = np.where(ex == 0, m * 2.0 ** -9, (8 + m) * np.exp2((ex - 10).astype(F64)))
    v = np.where((ex == 15) & (m == 7), np.nan, v)
    return sign * v


def encode_e4m3(t) -> np.ndarray:
    """Nearest representable value of t (fp32), ties to the even mantissa, saturating at +-448;
    -> code bytes (uint8).  The sign of zero is kept."""
    t = np.asarray(t, dtype=F32).astype(F64)
    a = np.minimum(np.abs(t), E4M3_MAX)
    _, ex = np.frexp(a)                         # a = f 2^ex, 0.5 <= f < 1  ->  floor(log2 a) = ex - 1
    E = np.maximum(ex - 1, -6)                  # below the smallest normal the subnormal spacing holds
    q = rne(a / np.exp2((E - 3).astype(F64)))   # multiples of the spacing 2^(E-3): 8..16 (normal), 0..8 (subnormal)
    up = q == 16                                # rounded up into the next binade
    E = np.where(up, E + 1, E)
    q = np.where(up, 8, q)
    normal = q >= 8
    field = np.where(normal, ((E + 7).astype(np.int64) << 3) | (q.astype(np.int64) - 8), q.astype(np.int64))
    field = np.minimum(field, 0x7E)             # 464 < a <= 448 cannot happen after the clamp; belt and braces
    sign = np.where(np.signbit(t), 0x80, 0)
    return (field | sign).astype(np.uint8)


# ------------------------------------------------------------------------------------ log2
def decode_log2(code) -> np.ndarray:
    """sign * 2^-e (float64); the zero code gives 0."""
    c = np.asarray(code).astype(np.uint8).astype(np.int64)
    e = c & 0x7F
    v = np.where(e == LOG2_ZERO, 0.0, np.exp2(-e.astype(F64)))
    return np.where(c & 0x80, -v, v)


def encode_log2(t) -> np.ndarray:
    """Nearest power of two of |t| (fp32) in the log domain, as 2^-e with 0 <= e <= 126; larger
    values saturate at e = 0, smaller ones and zero take the zero code.  -> code bytes (uint8)."""
    t = np.asarray(t, dtype=F32)
    a = np.abs(t)
    f, ex = np.frexp(a)                         # a = f 2^ex, 0.5 <= f < 1
    f2 = (f * F32(2.0)).astype(F32)             # 1 <= f2 < 2 (exact)
    k = (ex - 1) + (f2 >= SQRT2_F32)
    e = -k
    zero = (a == 0) | (e > 126)
    e = np.clip(e, 0, 126)
    field = np.where(zero, LOG2_ZERO, e).astype(np.int64)
    sign = np.where(np.signbit(t) & ~zero, 0x80, 0)
    return (field | sign).astype(np.uint8)


def encode(fmt, v, inv_s) -> np.ndarray:
    """t = fp32(v) * fp32(1/s), one fp32 multiply, then the format's rounding."""
    t = (np.asarray(v, dtype=F32) * F32(inv_s)).astype(F32)
    return encode_e4m3(t) if fmt == "e4m3" else encode_log2(t)


def decode(fmt, code) -> np.ndarray:
    return decode_e4m3(code) if fmt == "e4m3" else decode_log2(code)


def requant_real(acc, m) -> np.ndarray:
    """Real accumulator -> int8: clamp(rne(fp32(acc) * m), -128, 127)."""
    t = np.asarray(acc, dtype=F64).astype(F32) * F32(m)
    return np.clip(rne(t), QMIN, QMAX).astype(np.int8)


# ------------------------------------------------------------------------------------ mixer
def calibrate_xfmt(w, calib_u, fmt, x_percentile=99.999):
    """Quamba's calibration plus the format's scale of x.  Returns (qw, sc, xf)."""
    assert fmt in FORMATS
    qw, sc = calibrate(w, calib_u, x_percentile)
    x = np.asarray(fp_forward(w, calib_u)["x"], dtype=F64)
    if fmt == "e4m3":
        top = percentile_max(x, x_percentile)
        s = F32(top / E4M3_MAX) if top > 0.0 else F32(1.0)
    else:
        top = float(np.max(np.abs(x)))
        s = F32(top) if top > 0.0 else F32(1.0)
    d = {k: float(v) for k, v in sc.items()}
    xf = {
        "fmt": fmt, "s_x": s, "inv_s_x": F32(1.0 / float(s)),
        "m_x_dt": F32(float(s) * d["s_Wx"] / d["s_dtl"]), "m_x_B": F32(float(s) * d["s_Wx"] / d["s_B"]),
        "m_x_C": F32(float(s) * d["s_Wx"] / d["s_C"]),
    }
    return qw, sc, xf


def x_proj_real(x_code, W_x_q, fmt) -> np.ndarray:
    """acc[.., n] = sum_k W_q[n, k] value(x_code[.., k]) in float64."""
    v = decode(fmt, x_code)
    return v @ np.asarray(W_x_q).astype(F64).T


def _x_path(qw, sc, xf, x32, t):
    Di, R, N = _dims(qw)
    fmt = xf["fmt"]
    x_code = encode(fmt, x32, xf["inv_s_x"])
    lead = x_code.shape[:-1]
    acc_x = x_proj_real(x_code.reshape(-1, Di), qw["W_x"], fmt).reshape(*lead, R + 2 * N)
    dtl_q = requant_real(acc_x[..., :R], xf["m_x_dt"])
    B_q = requant_real(acc_x[..., R:R + N], xf["m_x_B"])
    C_q = requant_real(acc_x[..., R + N:], xf["m_x_C"])
    acc_dt = int_matmul(dtl_q.reshape(-1, R), qw["W_dt"]).reshape(*lead, Di)
    dt_q = requant_acc(acc_dt, sc["m_dt"])
    x_deq = (F32(xf["s_x"]) * decode(fmt, x_code).astype(F32)).astype(F32)
    t.update(x_code=x_code, acc_x=acc_x, dtl_q=dtl_q, B_q=B_q, C_q=C_q, acc_dt=acc_dt, dt_q=dt_q, x_deq=x_deq)
    return t


def _tail(qw, sc, t, z_q, h0):
    g, g16, h = q_scan(None, t["dt_q"], z_q, t["B_q"], t["C_q"], qw["A"], qw["D"], qw["dt_bias"], sc, h0,
                       x_values=t["x_deq"])
    gH, gH_q = q_hadamard_quant(g16, sc)
    acc_out, out = q_out_proj(gH_q, qw["W_outH"], sc)
    t.update(g=g, g16=g16, gH=gH, gH_q=gH_q, acc_out=acc_out, out=out, h=h)
    return t


def q_prefill_xfmt(qw, sc, xf, u=None, h0=None, u_q=None):
    """The quantized mixer with x in the format xf names, whole sequences from an empty conv
    history; arguments and results as `q_prefill`, plus xf."""
    Di, R, N = _dims(qw)
    t = _in_proj(qw, sc, u, u_q)
    xpre_q, z_q = t["xpre_q"], t["z_q"]
    Bt, L, _ = xpre_q.shape
    W = qw["conv_w"].shape[1]
    _x_path(qw, sc, xf, conv_prefill_silu(xpre_q, qw["conv_w"], qw["conv_b"], sc), t)
    _tail(qw, sc, t, z_q, h0)
    hist = np.zeros((Bt, W - 1, Di), dtype=F32)
    take = min(L, W - 1)
    hist[:, W - 1 - take:, :] = F32(sc["s_xpre"]) * xpre_q[:, L - take:, :].astype(F32)
    t["conv_state"] = np.ascontiguousarray(hist.transpose(0, 2, 1)).astype(np.float16)
    return t


def q_decode_xfmt(qw, sc, xf, u, ssm_state, conv_state, u_q=None):
    """One generation step with x in the format xf names; arguments and results as `q_decode`, plus xf."""
    t = _in_proj(qw, sc, None if u is None else np.asarray(u)[:, None, :],
                 None if u_q is None else np.asarray(u_q)[:, None, :])
    xpre_q, z_q = t["xpre_q"], t["z_q"]
    x32, new_state = conv_step_silu(xpre_q[:, 0, :], conv_state, qw["conv_w"], qw["conv_b"], sc)
    _x_path(qw, sc, xf, x32[:, None, :], t)
    _tail(qw, sc, t, z_q, ssm_state)
    t["conv_state"] = new_state
    return t
