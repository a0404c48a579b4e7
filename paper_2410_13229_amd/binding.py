"""ctypes binding of libquamba.so: argument marshalling only.

Tensors are passed as anything with ``data_ptr()`` (torch tensors on the GPU), a raw integer
address, or None.  Every function returns nothing and raises ``QuambaError`` when the
library reports a non-zero code.
"""
from __future__ import annotations

import ctypes as C
import os

__all__ = [
    "QuambaError", "Dims", "Scales", "QWeights", "FpWeights", "Taps", "lib", "lib_path",
    "SCALE_FIELDS", "scales_from_dict", "scales_to_dict", "make_qweights", "make_dims",
    "quamba_last_error", "quamba_workspace_bytes", "quamba_calibrate_workspace_bytes",
    "quamba_calibrate", "quamba_mixer_prefill", "quamba_mixer_prefill_q", "quamba_mixer_decode",
    "quamba_mixer_decode_q", "quamba_mixer_decode_noalloc", "quamba_add_rmsnorm_quant", "quamba_quantize_f16", "quamba_gemm_i8",
    "quamba_gemm_workspace_bytes", "quamba_conv_silu_quant", "quamba_conv_step", "quamba_scan_workspace_bytes",
    "quamba_scan_prefill", "quamba_scan_prefill_dtproj", "quamba_scan_step", "quamba_hadamard_quant",
    "Layer", "Model", "make_model", "quamba_model_workspace_bytes", "quamba_model_prefill", "quamba_model_decode",
    "quamba_model_generate", "quamba_calibrate_block", "quamba_embed", "quamba_final_norm", "quamba_lm_head", "quamba_argmax",
    "X_PERCENTILE", "X_MSE_CLIP", "quamba_calibrate_x_rule", "quamba_clip_search_workspace_bytes", "quamba_clip_search", "quamba_mixer_fp32",
    "Hadx", "HadxTaps", "HADX_FIELDS", "make_hadx", "hadx_to_dict", "quamba_calibrate_hadx", "quamba_hadx_workspace_bytes",
    "quamba_mixer_prefill_hadx", "quamba_mixer_decode_hadx", "quamba_hadamard_inverse",
    "XAsym", "XASYM_FIELDS", "make_xasym", "xasym_to_dict", "quamba_calibrate_xasym", "quamba_mixer_prefill_xasym",
    "quamba_mixer_decode_xasym",
    "XFmt", "XFMT_FIELDS", "XFMT_E4M3", "XFMT_LOG2", "make_xfmt", "xfmt_to_dict", "quamba_calibrate_xfmt",
    "quamba_mixer_prefill_xfmt", "quamba_mixer_decode_xfmt", "quamba_x_encode", "quamba_xfmt_proj",
    "quamba_xdyn_workspace_bytes", "quamba_mixer_prefill_xdyn", "quamba_mixer_decode_xdyn",
    "quamba_debug_set_gemm_variant", "quamba_debug_set_gemm_split", "quamba_debug_set_gemv_max_rows",
    "quamba_debug_set_fuse_dt", "quamba_debug_set_fuse_decode", "quamba_debug_set_scan_variant",
    "PROBE_FMA_F32", "PROBE_EXP_F32", "PROBE_SCAN_MIX", "PROBE_MFMA_I8", "PROBE_MFMA_I8_RANDOM",
    "PROBE_MUL_F32", "PROBE_FMA_EXP_INDEP", "PROBE_MIX_NOEXP", "PROBE_MIX_GROUPED",
    "quamba_probe_workspace_bytes", "quamba_probe_rate",
]

X_PERCENTILE, X_MSE_CLIP = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class QuambaError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"libquamba error {code}: {text}")
        self.code = code


def lib_path() -> str:
    return os.path.join(_HERE, "libquamba.so")


class Dims(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("d_model", "d_inner", "d_state", "dt_rank", "d_conv")]


SCALE_FIELDS = ("s_u", "s_xpre", "s_z", "s_x", "s_dtl", "s_B", "s_C", "s_dt", "s_y",
                "s_Win", "s_cw", "s_Wx", "s_Wdt", "s_A", "s_D", "s_WoutH",
                "inv_s_u", "m_in_x", "m_in_z", "m_conv", "inv_s_x", "m_x_dt", "m_x_B", "m_x_C",
                "m_dt", "inv_s_y", "m_out")


class Scales(C.Structure):
    _fields_ = [(n, C.c_float) for n in SCALE_FIELDS]


class FpWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("W_in", "conv_w", "conv_b", "W_x", "W_dt", "dt_bias",
                                          "A_log", "D", "W_out")]


class QWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("W_in", "conv_w", "W_x", "W_dt", "A", "D", "W_outH",
                                          "conv_b", "dt_bias")]


class Taps(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("u_q", "acc_in", "xz_q", "x_q", "acc_x", "dbc_q", "acc_dt",
                                          "dt_q", "y_f32", "g16", "gH_f32", "gH_q", "acc_out")]


HADX_FIELDS = ("s_xH", "s_WxH", "inv_s_xH", "m_xh_dt", "m_xh_B", "m_xh_C", "xhat_scale")


class Hadx(C.Structure):
    _fields_ = [("W_xH", C.c_void_p)] + [(n, C.c_float) for n in HADX_FIELDS]


class HadxTaps(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("x16", "xH_q", "xhat16")]


XASYM_FIELDS = ("s_x", "inv_s_x", "m_x_dt", "m_x_B", "m_x_C")


class XAsym(C.Structure):
    _fields_ = [("col_bias", C.c_void_p), ("zero_point", C.c_int32)] + [(n, C.c_float) for n in XASYM_FIELDS]


XFMT_FIELDS = ("s_x", "inv_s_x", "m_x_dt", "m_x_B", "m_x_C")
XFMT_E4M3, XFMT_LOG2 = 1, 2


class XFmt(C.Structure):
    _fields_ = [("W_x_bf16", C.c_void_p), ("format", C.c_int32)] + [(n, C.c_float) for n in XFMT_FIELDS]


class Layer(C.Structure):
    _fields_ = [("q", QWeights), ("s", Scales), ("norm_w", C.c_void_p)]


class Model(C.Structure):
    _fields_ = [("dims", Dims), ("n_layers", C.c_int), ("vocab", C.c_int), ("eps", C.c_float),
                ("embedding", C.c_void_p), ("norm_f", C.c_void_p), ("layers", C.POINTER(Layer))]


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return C.c_void_p(s)
    return C.c_void_p(s.cuda_stream)  # torch.cuda.Stream


def _struct_of_ptrs(cls, src):
    """Build a pointer struct from a dict / object of tensors (missing or None -> NULL)."""
    if src is None:
        return None
    if isinstance(src, cls):
        return src
    out = cls()
    for name, _ in cls._fields_:
        v = src.get(name) if isinstance(src, dict) else getattr(src, name, None)
        setattr(out, name, None if v is None else (v if isinstance(v, int) else v.data_ptr()))
    return out


def make_hadx(W_xH, values=None) -> Hadx:
    """Hadx struct over a device tensor W_xH (keep it alive) and, optionally, a dict of the scalars."""
    h = Hadx()
    h.W_xH = W_xH.data_ptr()
    for n in HADX_FIELDS:
        if values is not None:
            setattr(h, n, float(values[n]))
    return h


def hadx_to_dict(h: Hadx) -> dict:
    return {n: float(getattr(h, n)) for n in HADX_FIELDS}


def make_xasym(col_bias, values=None) -> XAsym:
    """XAsym struct over a device int32 tensor col_bias (keep it alive) and, optionally, a dict of the scalars."""
    a = XAsym()
    a.col_bias = col_bias.data_ptr()
    if values is not None:
        a.zero_point = int(values["zero_point"])
        for n in XASYM_FIELDS:
            setattr(a, n, float(values[n]))
    return a


def xasym_to_dict(a: XAsym) -> dict:
    d = {n: float(getattr(a, n)) for n in XASYM_FIELDS}
    d["zero_point"] = int(a.zero_point)
    return d


def make_xfmt(W_x_bf16, values=None) -> XFmt:
    """XFmt struct over a device int16 tensor W_x_bf16 (keep it alive) and, optionally, a dict of the scalars."""
    a = XFmt()
    a.W_x_bf16 = W_x_bf16.data_ptr()
    if values is not None:
        a.format = int(values["format"])
        for n in XFMT_FIELDS:
            setattr(a, n, float(values[n]))
    return a


def xfmt_to_dict(a: XFmt) -> dict:
    d = {n: float(getattr(a, n)) for n in XFMT_FIELDS}
    d["format"] = int(a.format)
    return d


def make_qweights(src) -> QWeights:
    """Pointer struct built once from a dict of device tensors (keep the dict alive)."""
    return _struct_of_ptrs(QWeights, src)


def make_dims(d) -> Dims:
    return _dims(d)


def make_model(dims, embedding, norm_f, layers, eps=1e-5) -> Model:
    """Model struct from device tensors: embedding fp16 [vocab, Dm], norm_f fp16 [Dm], layers a list of
    (qweights dict / QWeights, scales dict / Scales, norm_w fp16 [Dm]).  The struct keeps the layer array and
    the tensors alive through attributes of its own."""
    arr = (Layer * len(layers))()
    keep = [embedding, norm_f]
    for i, (qw, sc, nw) in enumerate(layers):
        arr[i].q = _struct_of_ptrs(QWeights, qw)
        arr[i].s = scales_from_dict(sc)
        arr[i].norm_w = nw.data_ptr()
        keep += [qw, nw]
    m = Model(_dims(dims), len(layers), int(embedding.shape[0]), float(eps), embedding.data_ptr(), norm_f.data_ptr(),
              C.cast(arr, C.POINTER(Layer)))
    m._keep = (arr, keep)
    return m


def scales_from_dict(d) -> Scales:
    if isinstance(d, Scales):
        return d
    s = Scales()
    for n in SCALE_FIELDS:
        setattr(s, n, float(d[n]))
    return s


def scales_to_dict(s: Scales) -> dict:
    return {n: getattr(s, n) for n in SCALE_FIELDS}


def _dims(d) -> Dims:
    if isinstance(d, Dims):
        return d
    if not hasattr(d, "d_model"):
        raise TypeError("dims must expose d_model, d_inner, d_state, dt_rank, d_conv")
    return Dims(int(d.d_model), int(d.d_inner), int(d.d_state), int(d.dt_rank), int(d.d_conv))


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise QuambaError(-100, f"{path} not found: build it with `python -m paper_2410_13229_amd.build`")
    try:  # a process that also uses PyTorch must end up with one HIP runtime: PyTorch's, loaded first
        import torch  # noqa: F401
    except ImportError:
        pass
    L = C.CDLL(path)
    vp, i, f, sz = C.c_void_p, C.c_int, C.c_float, C.c_size_t
    P = C.POINTER
    L.quamba_last_error.restype = C.c_char_p
    L.quamba_last_error.argtypes = []
    L.quamba_workspace_bytes.restype = sz
    L.quamba_workspace_bytes.argtypes = [P(Dims), i, i]
    L.quamba_calibrate_workspace_bytes.restype = sz
    L.quamba_calibrate_workspace_bytes.argtypes = [P(Dims), i, i]
    L.quamba_calibrate.argtypes = [P(Dims), P(FpWeights), vp, i, i, C.c_double, P(QWeights), P(Scales), vp, sz, vp]
    mix = [P(Dims), P(QWeights), P(Scales), vp, i, i, vp, vp, vp, P(Taps), vp, sz, vp]
    L.quamba_mixer_prefill.argtypes = mix
    L.quamba_mixer_prefill_q.argtypes = mix
    dec = [P(Dims), P(QWeights), P(Scales), vp, i, vp, vp, vp, P(Taps), vp, sz, vp]
    L.quamba_mixer_decode.argtypes = dec
    L.quamba_mixer_decode_q.argtypes = dec
    L.quamba_mixer_decode_noalloc.argtypes = [P(Dims), P(QWeights), P(Scales), vp, i, vp, vp, vp, P(Taps), vp]
    L.quamba_add_rmsnorm_quant.argtypes = [vp, vp, vp, f, f, vp, i, i, vp]
    L.quamba_quantize_f16.argtypes = [vp, vp, sz, f, vp]
    L.quamba_gemm_i8.argtypes = [vp, i, vp, i, i, i, i, i, i, P(C.c_float), vp, vp, i, vp, vp, sz, vp]
    L.quamba_gemm_workspace_bytes.restype = sz
    L.quamba_gemm_workspace_bytes.argtypes = [i, i, i]
    L.quamba_conv_silu_quant.argtypes = [vp, i, vp, vp, i, i, i, f, f, f, vp, vp, vp]
    L.quamba_conv_step.argtypes = [vp, i, vp, vp, i, i, f, f, f, vp, vp, vp]
    L.quamba_scan_workspace_bytes.restype = sz
    L.quamba_scan_workspace_bytes.argtypes = [i, i, i]
    L.quamba_scan_prefill.argtypes = [vp, vp, vp, i, vp, vp, i, vp, vp, vp, P(Scales), i, i, i, vp, vp, vp, vp, sz, vp]
    L.quamba_scan_prefill_dtproj.argtypes = [vp, vp, i, vp, i, f, vp, vp, i, vp, vp, i, vp, vp, vp, P(Scales), i, i,
                                             i, vp, vp, vp, vp, sz, vp]
    L.quamba_scan_step.argtypes = [vp, vp, vp, i, vp, vp, i, vp, vp, vp, P(Scales), i, i, vp, vp, vp, vp]
    L.quamba_hadamard_quant.argtypes = [vp, i, i, f, vp, vp, vp]
    L.quamba_calibrate_block.argtypes = [P(Dims), P(FpWeights), vp, f, vp, vp, i, i, C.c_double, P(QWeights), P(Scales),
                                         vp, sz, vp]
    L.quamba_calibrate_block.restype = C.c_int
    L.quamba_model_workspace_bytes.restype = sz
    L.quamba_model_workspace_bytes.argtypes = [P(Model), i, i]
    L.quamba_model_prefill.argtypes = [P(Model), vp, i, i, vp, vp, vp, vp, vp, sz, vp]
    L.quamba_model_decode.argtypes = [P(Model), vp, i, vp, vp, vp, vp, vp, sz, vp]
    L.quamba_model_generate.argtypes = [P(Model), vp, i, i, vp, vp, vp, vp, sz, i, vp]
    L.quamba_embed.argtypes = [vp, vp, i, i, i, vp, vp, vp]
    L.quamba_final_norm.argtypes = [vp, vp, vp, f, i, i, i, vp, vp]
    L.quamba_lm_head.argtypes = [vp, vp, i, i, i, vp, vp]
    L.quamba_argmax.argtypes = [vp, i, i, vp, vp]
    for name in ("quamba_model_prefill", "quamba_model_decode", "quamba_model_generate", "quamba_embed",
                 "quamba_final_norm", "quamba_lm_head", "quamba_argmax"):
        getattr(L, name).restype = C.c_int
    L.quamba_calibrate_x_rule.argtypes = [P(Dims), P(FpWeights), vp, i, i, i, C.c_double, P(QWeights), P(Scales), vp,
                                          sz, vp]
    L.quamba_clip_search_workspace_bytes.restype = sz
    L.quamba_clip_search_workspace_bytes.argtypes = []
    L.quamba_clip_search.argtypes = [vp, sz, i, i, P(C.c_double), P(C.c_int), vp, sz, vp]
    L.quamba_calibrate_hadx.argtypes = [P(Dims), P(FpWeights), vp, i, i, C.c_double, P(QWeights), P(Scales), P(Hadx), vp,
                                        sz, vp]
    L.quamba_hadx_workspace_bytes.restype = sz
    L.quamba_hadx_workspace_bytes.argtypes = [P(Dims), i, i]
    L.quamba_mixer_prefill_hadx.argtypes = [P(Dims), P(QWeights), P(Scales), P(Hadx), vp, i, i, vp, vp, vp, P(Taps),
                                            P(HadxTaps), vp, sz, vp]
    L.quamba_mixer_decode_hadx.argtypes = [P(Dims), P(QWeights), P(Scales), P(Hadx), vp, i, vp, vp, vp, P(Taps),
                                           P(HadxTaps), vp, sz, vp]
    L.quamba_hadamard_inverse.argtypes = [vp, i, i, f, vp, vp]
    for name in ("quamba_calibrate_hadx", "quamba_mixer_prefill_hadx", "quamba_mixer_decode_hadx",
                 "quamba_hadamard_inverse"):
        getattr(L, name).restype = C.c_int
    L.quamba_calibrate_xasym.argtypes = [P(Dims), P(FpWeights), vp, i, i, C.c_double, P(QWeights), P(Scales), P(XAsym),
                                         vp, sz, vp]
    L.quamba_mixer_prefill_xasym.argtypes = [P(Dims), P(QWeights), P(Scales), P(XAsym), vp, i, i, vp, vp, vp, P(Taps),
                                             vp, sz, vp]
    L.quamba_mixer_decode_xasym.argtypes = [P(Dims), P(QWeights), P(Scales), P(XAsym), vp, i, vp, vp, vp, P(Taps),
                                            vp, sz, vp]
    for name in ("quamba_calibrate_xasym", "quamba_mixer_prefill_xasym", "quamba_mixer_decode_xasym"):
        getattr(L, name).restype = C.c_int
    L.quamba_calibrate_xfmt.argtypes = [P(Dims), P(FpWeights), vp, i, i, i, C.c_double, P(QWeights), P(Scales), P(XFmt),
                                        vp, sz, vp]
    L.quamba_mixer_prefill_xfmt.argtypes = [P(Dims), P(QWeights), P(Scales), P(XFmt), vp, i, i, vp, vp, vp, P(Taps),
                                            vp, sz, vp]
    L.quamba_mixer_decode_xfmt.argtypes = [P(Dims), P(QWeights), P(Scales), P(XFmt), vp, i, vp, vp, vp, P(Taps),
                                           vp, sz, vp]
    L.quamba_x_encode.argtypes = [i, vp, sz, f, vp, vp]
    L.quamba_xfmt_proj.argtypes = [i, vp, i, i, i, vp, i, i, P(C.c_float), vp, vp, vp, sz, vp]
    for name in ("quamba_calibrate_xfmt", "quamba_mixer_prefill_xfmt", "quamba_mixer_decode_xfmt", "quamba_x_encode",
                 "quamba_xfmt_proj"):
        getattr(L, name).restype = C.c_int
    L.quamba_xdyn_workspace_bytes.restype = sz
    L.quamba_xdyn_workspace_bytes.argtypes = [P(Dims), i, i]
    L.quamba_mixer_prefill_xdyn.argtypes = [P(Dims), P(QWeights), P(Scales), vp, i, i, vp, vp, vp, P(Taps), vp, vp, vp, sz, vp]
    L.quamba_mixer_decode_xdyn.argtypes = [P(Dims), P(QWeights), P(Scales), vp, i, vp, vp, vp, P(Taps), vp, vp, vp, sz, vp]
    for name in ("quamba_mixer_prefill_xdyn", "quamba_mixer_decode_xdyn"):
        getattr(L, name).restype = C.c_int
    L.quamba_mixer_fp32.argtypes = [P(Dims), P(FpWeights), vp, i, i, vp, vp, sz, vp]
    for name in ("quamba_calibrate_x_rule", "quamba_clip_search", "quamba_mixer_fp32"):
        getattr(L, name).restype = C.c_int
    for name in ("quamba_calibrate", "quamba_mixer_prefill", "quamba_mixer_prefill_q", "quamba_mixer_decode",
                 "quamba_mixer_decode_q", "quamba_mixer_decode_noalloc", "quamba_add_rmsnorm_quant",
                 "quamba_quantize_f16", "quamba_gemm_i8",
                 "quamba_conv_silu_quant", "quamba_conv_step", "quamba_scan_prefill", "quamba_scan_step",
                 "quamba_scan_prefill_dtproj", "quamba_hadamard_quant"):
        getattr(L, name).restype = C.c_int
    for name in ("quamba_debug_set_gemm_variant", "quamba_debug_set_gemm_split", "quamba_debug_set_gemv_max_rows",
                 "quamba_debug_set_fuse_dt", "quamba_debug_set_fuse_decode", "quamba_debug_set_scan_variant"):
        getattr(L, name).argtypes = [i]
        getattr(L, name).restype = None
    L.quamba_probe_workspace_bytes.restype = sz
    L.quamba_probe_workspace_bytes.argtypes = [i]
    L.quamba_probe_rate.restype = C.c_int
    L.quamba_probe_rate.argtypes = [i, i, i, P(C.c_double), vp, sz, vp]
    _LIB = L
    return L


def _check(rc):
    if rc != 0:
        raise QuambaError(rc, lib().quamba_last_error().decode())


def _nbytes(ws):
    return 0 if ws is None else ws.numel() * ws.element_size()


def quamba_last_error() -> str:
    return lib().quamba_last_error().decode()


def quamba_workspace_bytes(dims, batch, L) -> int:
    return int(lib().quamba_workspace_bytes(C.byref(_dims(dims)), batch, L))


def quamba_calibrate_workspace_bytes(dims, nb, Lc) -> int:
    return int(lib().quamba_calibrate_workspace_bytes(C.byref(_dims(dims)), nb, Lc))


def quamba_calibrate(dims, fp_weights, calib_u, nb, Lc, x_percentile, out_q, ws, stream=None) -> Scales:
    """Returns the filled Scales struct; `out_q` (dict of preallocated tensors) is written on the device."""
    fw = _struct_of_ptrs(FpWeights, fp_weights)
    oq = _struct_of_ptrs(QWeights, out_q)
    sc = Scales()
    _check(lib().quamba_calibrate(C.byref(_dims(dims)), C.byref(fw), _ptr(calib_u), nb, Lc, float(x_percentile),
                                  C.byref(oq), C.byref(sc), _ptr(ws), _nbytes(ws), _stream(stream)))
    return sc


def quamba_calibrate_x_rule(dims, fp_weights, calib_u, nb, Lc, x_rule, x_percentile, out_q, ws, stream=None) -> Scales:
    fw = _struct_of_ptrs(FpWeights, fp_weights)
    oq = _struct_of_ptrs(QWeights, out_q)
    sc = Scales()
    _check(lib().quamba_calibrate_x_rule(C.byref(_dims(dims)), C.byref(fw), _ptr(calib_u), nb, Lc, int(x_rule),
                                         float(x_percentile), C.byref(oq), C.byref(sc), _ptr(ws), _nbytes(ws),
                                         _stream(stream)))
    return sc


def quamba_mixer_fp32(dims, fp_weights, u, nb, L, out, ws, stream=None):
    fw = _struct_of_ptrs(FpWeights, fp_weights)
    _check(lib().quamba_mixer_fp32(C.byref(_dims(dims)), C.byref(fw), _ptr(u), nb, L, _ptr(out), _ptr(ws), _nbytes(ws),
                                   _stream(stream)))


def quamba_calibrate_hadx(dims, fp_weights, calib_u, nb, Lc, x_percentile, out_q, W_xH, ws, stream=None):
    """Returns (Scales, Hadx); `out_q` and `W_xH` (preallocated device tensors) are written on the device."""
    fw = _struct_of_ptrs(FpWeights, fp_weights)
    oq = _struct_of_ptrs(QWeights, out_q)
    sc, hx = Scales(), make_hadx(W_xH)
    _check(lib().quamba_calibrate_hadx(C.byref(_dims(dims)), C.byref(fw), _ptr(calib_u), nb, Lc, float(x_percentile),
                                       C.byref(oq), C.byref(sc), C.byref(hx), _ptr(ws), _nbytes(ws), _stream(stream)))
    return sc, hx


def quamba_hadx_workspace_bytes(dims, batch, L) -> int:
    return int(lib().quamba_hadx_workspace_bytes(C.byref(_dims(dims)), batch, L))


def _hadx_taps(t):
    t = _struct_of_ptrs(HadxTaps, t)
    return None if t is None else C.byref(t)


def quamba_mixer_prefill_hadx(dims, qw, sc, hx, u, Bt, L, out, ssm_state, conv_state, taps, hx_taps, ws, stream=None):
    _check(lib().quamba_mixer_prefill_hadx(C.byref(_dims(dims)), C.byref(_struct_of_ptrs(QWeights, qw)),
                                           C.byref(scales_from_dict(sc)), C.byref(hx), _ptr(u), Bt, L, _ptr(out),
                                           _ptr(ssm_state), _ptr(conv_state), _taps(taps), _hadx_taps(hx_taps),
                                           _ptr(ws), _nbytes(ws), _stream(stream)))


def quamba_mixer_decode_hadx(dims, qw, sc, hx, u, Bt, out, ssm_state, conv_state, taps, hx_taps, ws, stream=None):
    _check(lib().quamba_mixer_decode_hadx(C.byref(_dims(dims)), C.byref(_struct_of_ptrs(QWeights, qw)),
                                          C.byref(scales_from_dict(sc)), C.byref(hx), _ptr(u), Bt, _ptr(out),
                                          _ptr(ssm_state), _ptr(conv_state), _taps(taps), _hadx_taps(hx_taps),
                                          _ptr(ws), _nbytes(ws), _stream(stream)))


def quamba_hadamard_inverse(xH_q, M, n, scale, x_hat, stream=None):
    _check(lib().quamba_hadamard_inverse(_ptr(xH_q), M, n, float(scale), _ptr(x_hat), _stream(stream)))


def quamba_calibrate_xasym(dims, fp_weights, calib_u, nb, Lc, x_percentile, out_q, col_bias, ws, stream=None):
    """Returns (Scales, XAsym); `out_q` and `col_bias` (preallocated device tensors) are written on the device."""
    fw = _struct_of_ptrs(FpWeights, fp_weights)
    oq = _struct_of_ptrs(QWeights, out_q)
    sc, xa = Scales(), make_xasym(col_bias)
    _check(lib().quamba_calibrate_xasym(C.byref(_dims(dims)), C.byref(fw), _ptr(calib_u), nb, Lc, float(x_percentile),
                                        C.byref(oq), C.byref(sc), C.byref(xa), _ptr(ws), _nbytes(ws), _stream(stream)))
    return sc, xa


def quamba_mixer_prefill_xasym(dims, qw, sc, xa, u, Bt, L, out, ssm_state, conv_state, taps, ws, stream=None):
    _check(lib().quamba_mixer_prefill_xasym(C.byref(_dims(dims)), C.byref(_struct_of_ptrs(QWeights, qw)),
                                            C.byref(scales_from_dict(sc)), C.byref(xa), _ptr(u), Bt, L, _ptr(out),
                                            _ptr(ssm_state), _ptr(conv_state), _taps(taps), _ptr(ws), _nbytes(ws),
                                            _stream(stream)))


def quamba_mixer_decode_xasym(dims, qw, sc, xa, u, Bt, out, ssm_state, conv_state, taps, ws, stream=None):
    _check(lib().quamba_mixer_decode_xasym(C.byref(_dims(dims)), C.byref(_struct_of_ptrs(QWeights, qw)),
                                           C.byref(scales_from_dict(sc)), C.byref(xa), _ptr(u), Bt, _ptr(out),
                                           _ptr(ssm_state), _ptr(conv_state), _taps(taps), _ptr(ws), _nbytes(ws),
                                           _stream(stream)))


def quamba_calibrate_xfmt(dims, fp_weights, calib_u, nb, Lc, fmt, x_percentile, out_q, W_x_bf16, ws, stream=None):
    """Returns (Scales, XFmt); `out_q` and `W_x_bf16` (preallocated device tensors) are written on the device."""
    fw = _struct_of_ptrs(FpWeights, fp_weights)
    oq = _struct_of_ptrs(QWeights, out_q)
    sc, xf = Scales(), make_xfmt(W_x_bf16)
    _check(lib().quamba_calibrate_xfmt(C.byref(_dims(dims)), C.byref(fw), _ptr(calib_u), nb, Lc, int(fmt),
                                       float(x_percentile), C.byref(oq), C.byref(sc), C.byref(xf), _ptr(ws),
                                       _nbytes(ws), _stream(stream)))
    return sc, xf


def quamba_mixer_prefill_xfmt(dims, qw, sc, xf, u, Bt, L, out, ssm_state, conv_state, taps, ws, stream=None):
    _check(lib().quamba_mixer_prefill_xfmt(C.byref(_dims(dims)), C.byref(_struct_of_ptrs(QWeights, qw)),
                                           C.byref(scales_from_dict(sc)), C.byref(xf), _ptr(u), Bt, L, _ptr(out),
                                           _ptr(ssm_state), _ptr(conv_state), _taps(taps), _ptr(ws), _nbytes(ws),
                                           _stream(stream)))


def quamba_mixer_decode_xfmt(dims, qw, sc, xf, u, Bt, out, ssm_state, conv_state, taps, ws, stream=None):
    _check(lib().quamba_mixer_decode_xfmt(C.byref(_dims(dims)), C.byref(_struct_of_ptrs(QWeights, qw)),
                                          C.byref(scales_from_dict(sc)), C.byref(xf), _ptr(u), Bt, _ptr(out),
                                          _ptr(ssm_state), _ptr(conv_state), _taps(taps), _ptr(ws), _nbytes(ws),
                                          _stream(stream)))


def quamba_xdyn_workspace_bytes(dims, batch, L) -> int:
    return int(lib().quamba_xdyn_workspace_bytes(C.byref(_dims(dims)), batch, L))


def quamba_mixer_prefill_xdyn(dims, qw, sc, u, Bt, L, out, ssm_state, conv_state, taps, s_x_out, x16_out, ws, stream=None):
    _check(lib().quamba_mixer_prefill_xdyn(C.byref(_dims(dims)), C.byref(_struct_of_ptrs(QWeights, qw)),
                                           C.byref(scales_from_dict(sc)), _ptr(u), Bt, L, _ptr(out), _ptr(ssm_state),
                                           _ptr(conv_state), _taps(taps), _ptr(s_x_out), _ptr(x16_out), _ptr(ws),
                                           _nbytes(ws), _stream(stream)))


def quamba_mixer_decode_xdyn(dims, qw, sc, u, Bt, out, ssm_state, conv_state, taps, s_x_out, x16_out, ws, stream=None):
    _check(lib().quamba_mixer_decode_xdyn(C.byref(_dims(dims)), C.byref(_struct_of_ptrs(QWeights, qw)),
                                          C.byref(scales_from_dict(sc)), _ptr(u), Bt, _ptr(out), _ptr(ssm_state),
                                          _ptr(conv_state), _taps(taps), _ptr(s_x_out), _ptr(x16_out), _ptr(ws),
                                          _nbytes(ws), _stream(stream)))


def quamba_x_encode(fmt, v, n, inv_s, codes, stream=None):
    _check(lib().quamba_x_encode(int(fmt), _ptr(v), n, float(inv_s), _ptr(codes), _stream(stream)))


def quamba_xfmt_proj(fmt, x_code, M, N, K, W_bf16, e0, e1, mult, out_q, acc_f32, ws=None, stream=None):
    m = (C.c_float * 3)(*[float(v) for v in mult])
    _check(lib().quamba_xfmt_proj(int(fmt), _ptr(x_code), M, N, K, _ptr(W_bf16), e0, e1, m, _ptr(out_q), _ptr(acc_f32),
                                  _ptr(ws), _nbytes(ws), _stream(stream)))


def quamba_clip_search_workspace_bytes() -> int:
    return int(lib().quamba_clip_search_workspace_bytes())


def quamba_clip_search(x, n, bits, max_iters, ws, stream=None):
    """Returns (clip, updates made)."""
    clip, iters = C.c_double(0.0), C.c_int(0)
    _check(lib().quamba_clip_search(_ptr(x), n, bits, max_iters, C.byref(clip), C.byref(iters), _ptr(ws), _nbytes(ws),
                                    _stream(stream)))
    return clip.value, iters.value


def _taps(t):
    t = _struct_of_ptrs(Taps, t)
    return None if t is None else C.byref(t)


def quamba_mixer_prefill(dims, qw, sc, u, Bt, L, out, ssm_state, conv_state, taps, ws, stream=None):
    _check(lib().quamba_mixer_prefill(C.byref(_dims(dims)), C.byref(_struct_of_ptrs(QWeights, qw)),
                                      C.byref(scales_from_dict(sc)), _ptr(u), Bt, L, _ptr(out), _ptr(ssm_state),
                                      _ptr(conv_state), _taps(taps), _ptr(ws), _nbytes(ws), _stream(stream)))


def quamba_mixer_prefill_q(dims, qw, sc, u_q, Bt, L, out, ssm_state, conv_state, taps, ws, stream=None):
    _check(lib().quamba_mixer_prefill_q(C.byref(_dims(dims)), C.byref(_struct_of_ptrs(QWeights, qw)),
                                        C.byref(scales_from_dict(sc)), _ptr(u_q), Bt, L, _ptr(out),
                                        _ptr(ssm_state), _ptr(conv_state), _taps(taps), _ptr(ws), _nbytes(ws),
                                        _stream(stream)))


def quamba_mixer_decode(dims, qw, sc, u, Bt, out, ssm_state, conv_state, taps, ws, stream=None):
    _check(lib().quamba_mixer_decode(C.byref(_dims(dims)), C.byref(_struct_of_ptrs(QWeights, qw)),
                                     C.byref(scales_from_dict(sc)), _ptr(u), Bt, _ptr(out), _ptr(ssm_state),
                                     _ptr(conv_state), _taps(taps), _ptr(ws), _nbytes(ws), _stream(stream)))


def quamba_mixer_decode_noalloc(dims, qw, sc, u, Bt, out, ssm_state, conv_state, taps, stream=None):
    _check(lib().quamba_mixer_decode_noalloc(C.byref(_dims(dims)), C.byref(_struct_of_ptrs(QWeights, qw)),
                                             C.byref(scales_from_dict(sc)), _ptr(u), Bt, _ptr(out), _ptr(ssm_state),
                                             _ptr(conv_state), _taps(taps), _stream(stream)))


def quamba_mixer_decode_q(dims, qw, sc, u_q, Bt, out, ssm_state, conv_state, taps, ws, stream=None):
    _check(lib().quamba_mixer_decode_q(C.byref(_dims(dims)), C.byref(_struct_of_ptrs(QWeights, qw)),
                                       C.byref(scales_from_dict(sc)), _ptr(u_q), Bt, _ptr(out), _ptr(ssm_state),
                                       _ptr(conv_state), _taps(taps), _ptr(ws), _nbytes(ws), _stream(stream)))


def quamba_add_rmsnorm_quant(x_out, res, weight, eps, inv_s, u_q, M, Dm, stream=None):
    _check(lib().quamba_add_rmsnorm_quant(_ptr(x_out), _ptr(res), _ptr(weight), float(eps), float(inv_s),
                                          _ptr(u_q), M, Dm, _stream(stream)))


def quamba_quantize_f16(x, q, n, inv_s, stream=None):
    _check(lib().quamba_quantize_f16(_ptr(x), _ptr(q), n, float(inv_s), _stream(stream)))


def quamba_gemm_workspace_bytes(M, N, K) -> int:
    return int(lib().quamba_gemm_workspace_bytes(M, N, K))


def quamba_gemm_i8(A, lda, Wt, ldw, M, N, K, col_end0, col_end1, mult, out_i8, out_f16, ldo, acc_out, ws=None,
                   stream=None):
    m = (C.c_float * 3)(*[float(v) for v in mult])
    _check(lib().quamba_gemm_i8(_ptr(A), lda, _ptr(Wt), ldw, M, N, K, col_end0, col_end1, m, _ptr(out_i8),
                                _ptr(out_f16), ldo, _ptr(acc_out), _ptr(ws), _nbytes(ws), _stream(stream)))


def quamba_conv_silu_quant(xpre_q, ldx, w_q, conv_b, Bt, L, Di, m_conv, inv_s_x, s_xpre, x_q, conv_state,
                           stream=None):
    _check(lib().quamba_conv_silu_quant(_ptr(xpre_q), ldx, _ptr(w_q), _ptr(conv_b), Bt, L, Di, float(m_conv),
                                        float(inv_s_x), float(s_xpre), _ptr(x_q), _ptr(conv_state),
                                        _stream(stream)))


def quamba_conv_step(xpre_q, ldx, w_q, conv_b, Bt, Di, s_cw, s_xpre, inv_s_x, x_q, conv_state, stream=None):
    _check(lib().quamba_conv_step(_ptr(xpre_q), ldx, _ptr(w_q), _ptr(conv_b), Bt, Di, float(s_cw), float(s_xpre),
                                  float(inv_s_x), _ptr(x_q), _ptr(conv_state), _stream(stream)))


def quamba_scan_workspace_bytes(Bt, L, Di) -> int:
    return int(lib().quamba_scan_workspace_bytes(Bt, L, Di))


def quamba_scan_prefill(x_q, dt_q, z_q, ldz, B_q, C_q, ldbc, A_q, D_q, dt_bias, sc, Bt, L, Di, g16, y_f32,
                        ssm_state, ws, stream=None):
    _check(lib().quamba_scan_prefill(_ptr(x_q), _ptr(dt_q), _ptr(z_q), ldz, _ptr(B_q), _ptr(C_q), ldbc, _ptr(A_q),
                                     _ptr(D_q), _ptr(dt_bias), C.byref(scales_from_dict(sc)), Bt, L, Di,
                                     _ptr(g16), _ptr(y_f32), _ptr(ssm_state), _ptr(ws), _nbytes(ws),
                                     _stream(stream)))


def quamba_scan_prefill_dtproj(x_q, dtlow_q, lddl, W_dt_q, R, m_dt, dt_q, z_q, ldz, B_q, C_q, ldbc, A_q, D_q, dt_bias,
                               sc, Bt, L, Di, g16, y_f32, ssm_state, ws, stream=None):
    _check(lib().quamba_scan_prefill_dtproj(_ptr(x_q), _ptr(dtlow_q), lddl, _ptr(W_dt_q), R, float(m_dt), _ptr(dt_q),
                                            _ptr(z_q), ldz, _ptr(B_q), _ptr(C_q), ldbc, _ptr(A_q), _ptr(D_q),
                                            _ptr(dt_bias), C.byref(scales_from_dict(sc)), Bt, L, Di, _ptr(g16),
                                            _ptr(y_f32), _ptr(ssm_state), _ptr(ws), _nbytes(ws), _stream(stream)))


def quamba_scan_step(x_q, dt_q, z_q, ldz, B_q, C_q, ldbc, A_q, D_q, dt_bias, sc, Bt, Di, g16, y_f32, ssm_state,
                     stream=None):
    _check(lib().quamba_scan_step(_ptr(x_q), _ptr(dt_q), _ptr(z_q), ldz, _ptr(B_q), _ptr(C_q), ldbc, _ptr(A_q),
                                  _ptr(D_q), _ptr(dt_bias), C.byref(scales_from_dict(sc)), Bt, Di, _ptr(g16),
                                  _ptr(y_f32), _ptr(ssm_state), _stream(stream)))


def quamba_hadamard_quant(g, M, n, inv_s_y, yH_q, yH_f32, stream=None):
    _check(lib().quamba_hadamard_quant(_ptr(g), M, n, float(inv_s_y), _ptr(yH_q), _ptr(yH_f32), _stream(stream)))


def quamba_model_workspace_bytes(model, batch, L) -> int:
    return int(lib().quamba_model_workspace_bytes(C.byref(model), batch, L))


def quamba_model_prefill(model, tokens, Bt, L, logits, next_token, ssm_states, conv_states, ws, stream=None):
    _check(lib().quamba_model_prefill(C.byref(model), _ptr(tokens), Bt, L, _ptr(logits), _ptr(next_token),
                                      _ptr(ssm_states), _ptr(conv_states), _ptr(ws), _nbytes(ws), _stream(stream)))


def quamba_model_decode(model, tokens, Bt, logits, next_token, ssm_states, conv_states, ws, stream=None):
    _check(lib().quamba_model_decode(C.byref(model), _ptr(tokens), Bt, _ptr(logits), _ptr(next_token),
                                     _ptr(ssm_states), _ptr(conv_states), _ptr(ws), _nbytes(ws), _stream(stream)))


def quamba_model_generate(model, first_tokens, Bt, n_new, tokens_out, ssm_states, conv_states, ws, use_graph=False,
                          stream=None):
    _check(lib().quamba_model_generate(C.byref(model), _ptr(first_tokens), Bt, n_new, _ptr(tokens_out),
                                       _ptr(ssm_states), _ptr(conv_states), _ptr(ws), _nbytes(ws),
                                       1 if use_graph else 0, _stream(stream)))


def quamba_embed(embedding, tokens, M, Dm, vocab, res, out, stream=None):
    _check(lib().quamba_embed(_ptr(embedding), _ptr(tokens), M, Dm, vocab, _ptr(res), _ptr(out), _stream(stream)))


def quamba_final_norm(out, res, weight, eps, Bt, L, Dm, y, stream=None):
    _check(lib().quamba_final_norm(_ptr(out), _ptr(res), _ptr(weight), float(eps), Bt, L, Dm, _ptr(y),
                                   _stream(stream)))


def quamba_lm_head(y, embedding, Bt, vocab, Dm, logits, stream=None):
    _check(lib().quamba_lm_head(_ptr(y), _ptr(embedding), Bt, vocab, Dm, _ptr(logits), _stream(stream)))


def quamba_argmax(logits, Bt, vocab, next_token, stream=None):
    _check(lib().quamba_argmax(_ptr(logits), Bt, vocab, _ptr(next_token), _stream(stream)))


def quamba_calibrate_block(dims, fp_weights, norm_w, eps, res, out, nb, Lc, x_percentile, out_q, ws, stream=None) -> Scales:
    """One block of a stack: advances the fp32 residual stream (res, out) and returns the block's Scales."""
    fw = _struct_of_ptrs(FpWeights, fp_weights)
    oq = _struct_of_ptrs(QWeights, out_q)
    sc = Scales()
    _check(lib().quamba_calibrate_block(C.byref(_dims(dims)), C.byref(fw), _ptr(norm_w), float(eps), _ptr(res), _ptr(out),
                                        nb, Lc, float(x_percentile), C.byref(oq), C.byref(sc), _ptr(ws), _nbytes(ws),
                                        _stream(stream)))
    return sc


# ---- tuning hooks (process-wide switches between kernels that compute the same thing)
def quamba_debug_set_gemm_variant(v):
    lib().quamba_debug_set_gemm_variant(int(v))


def quamba_debug_set_gemm_split(v):
    lib().quamba_debug_set_gemm_split(int(v))


def quamba_debug_set_gemv_max_rows(v):
    lib().quamba_debug_set_gemv_max_rows(int(v))


def quamba_debug_set_fuse_dt(v):
    lib().quamba_debug_set_fuse_dt(int(v))


def quamba_debug_set_fuse_decode(v):
    lib().quamba_debug_set_fuse_decode(int(v))


def quamba_debug_set_scan_variant(v):
    lib().quamba_debug_set_scan_variant(int(v))


# ---- diagnostics: instruction-rate probes
PROBE_FMA_F32, PROBE_EXP_F32, PROBE_SCAN_MIX, PROBE_MFMA_I8, PROBE_MFMA_I8_RANDOM = 0, 1, 2, 3, 4
PROBE_MUL_F32, PROBE_FMA_EXP_INDEP, PROBE_MIX_NOEXP, PROBE_MIX_GROUPED = 5, 6, 7, 8


def quamba_probe_workspace_bytes(waves_per_simd) -> int:
    return int(lib().quamba_probe_workspace_bytes(int(waves_per_simd)))


def quamba_probe_rate(probe, waves_per_simd, iters, ws, stream=None) -> float:
    """Enqueues one probe launch; returns the number of counted instructions of that launch."""
    n = C.c_double(0.0)
    _check(lib().quamba_probe_rate(int(probe), int(waves_per_simd), int(iters), C.byref(n), _ptr(ws), _nbytes(ws),
                                   _stream(stream)))
    return n.value
