"""ctypes binding of the CPU oracle (liblstm_int_oracle.so).

TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT.  Only tests, the smoke check
and the benchmark's cpu_baseline leg may import this package; the HIP library
and its Python binding never do, and this package never imports them.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# LSTM_INT_ORACLE_LIB selects another build of the same source (the sanitized one of oracle/build.py)
_LIB_PATH = os.environ.get("LSTM_INT_ORACLE_LIB") or os.path.join(_HERE, "liblstm_int_oracle.so")

CIFG, PEEPHOLE, LAYER_NORM, PROJECTION = 1, 2, 4, 8
OK, INVALID_ARG, UNSUPPORTED, BAD_RANGE, NOMEM = 0, -1, -2, -3, -4

_fp = C.POINTER(C.c_float)


class _LayerParams(C.Structure):
    _fields_ = [
        ("input_size", C.c_int32), ("num_cells", C.c_int32), ("output_size", C.c_int32),
        ("flags", C.c_uint32),
        ("W", _fp * 4), ("R", _fp * 4), ("b", _fp * 4), ("P", _fp * 3), ("Lw", _fp * 4),
        ("Wproj", _fp), ("bproj", _fp),
        ("x_min", C.c_float), ("x_max", C.c_float), ("h_min", C.c_float), ("h_max", C.c_float),
        ("m_min", C.c_float), ("m_max", C.c_float), ("c_absmax", C.c_float),
        ("g_absmax", C.c_float * 4),
    ]


class _LayerQuant(C.Structure):
    _fields_ = [
        ("I", C.c_int32), ("N", C.c_int32), ("H", C.c_int32), ("G", C.c_int32),
        ("flags", C.c_uint32), ("m_c", C.c_int32),
        ("zp_x", C.c_int32), ("zp_h", C.c_int32), ("zp_m", C.c_int32),
        ("s_x", C.c_double), ("s_h", C.c_double), ("s_m", C.c_double), ("s_c", C.c_double),
        ("s_Wp", C.c_double),
        ("s_W", C.c_double * 4), ("s_R", C.c_double * 4), ("s_P", C.c_double * 3),
        ("s_L", C.c_double * 4), ("s_g", C.c_double * 4),
        ("Mx", C.c_int32 * 4), ("ex", C.c_int32 * 4),
        ("Mh", C.c_int32 * 4), ("eh", C.c_int32 * 4),
        ("Mc", C.c_int32 * 3), ("ec", C.c_int32 * 3),
        ("Mln", C.c_int32 * 4), ("eln", C.c_int32 * 4),
        ("Mm", C.c_int32), ("em", C.c_int32), ("Mp", C.c_int32), ("ep", C.c_int32),
        ("Wq", C.POINTER(C.c_int8)), ("Rq", C.POINTER(C.c_int8)),
        ("qb", C.POINTER(C.c_int32)), ("Pq", C.POINTER(C.c_int16)),
        ("Lq", C.POINTER(C.c_int16)), ("Wpq", C.POINTER(C.c_int8)),
        ("qbp", C.POINTER(C.c_int32)), ("bx_fold", C.POINTER(C.c_int32)),
        ("bh_fold", C.POINTER(C.c_int32)), ("bp_fold", C.POINTER(C.c_int32)),
    ]


class _Trace(C.Structure):
    _fields_ = [("layer", C.c_int32)] + [
        (n, C.c_void_p) for n in ("tx", "th", "g", "ln", "act", "c", "m", "h")
    ]


class _FloatStats(C.Structure):
    _fields_ = [(n, C.c_double) for n in
                ("x_min", "x_max", "h_min", "h_max", "m_min", "m_max", "c_absmax")] + [
        ("g_absmax", C.c_double * 4)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build()
        L = C.CDLL(_LIB_PATH)
        L.orc_rhu.restype = C.c_int64
        L.orc_rhu.argtypes = [C.c_int64, C.c_int64]
        L.orc_rsh_r.restype = C.c_int64
        L.orc_rsh_r.argtypes = [C.c_int64, C.c_int]
        L.orc_rescale.restype = C.c_int32
        L.orc_rescale.argtypes = [C.c_int64, C.c_int32, C.c_int]
        L.orc_quantize_multiplier.restype = C.c_int
        L.orc_quantize_multiplier.argtypes = [C.c_double, C.POINTER(C.c_int32), C.POINTER(C.c_int)]
        L.orc_isqrt.restype = C.c_int64
        L.orc_isqrt.argtypes = [C.c_int64]
        L.orc_expneg.restype = C.c_int64
        L.orc_expneg.argtypes = [C.c_int64]
        L.orc_int_sigmoid.restype = C.c_int32
        L.orc_int_sigmoid.argtypes = [C.c_int32, C.c_int]
        L.orc_int_tanh.restype = C.c_int32
        L.orc_int_tanh.argtypes = [C.c_int32, C.c_int]
        L.orc_int_layernorm.restype = C.c_int
        L.orc_int_layernorm.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int32,
                                        C.c_int, C.c_void_p]
        L.orc_prepare.restype = C.c_int
        L.orc_prepare.argtypes = [C.POINTER(_LayerParams), C.c_int32, C.POINTER(C.c_void_p)]
        L.orc_destroy.restype = None
        L.orc_destroy.argtypes = [C.c_void_p]
        L.orc_get_layer.restype = C.POINTER(_LayerQuant)
        L.orc_get_layer.argtypes = [C.c_void_p, C.c_int32]
        L.orc_forward.restype = C.c_int
        L.orc_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                  C.c_void_p, C.c_void_p, C.POINTER(_Trace), C.c_int, C.c_int]
        L.orc_float_forward.restype = C.c_int
        L.orc_float_forward.argtypes = [C.POINTER(_LayerParams), C.c_int32, C.c_void_p, C.c_int32,
                                        C.c_int32, C.c_void_p, C.POINTER(_FloatStats), C.c_int]
        L.orc_max_threads.restype = C.c_int
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"oracle {what} failed with code {code}")
        self.code = code


# ---------------------------------------------------------------- primitives
def rhu(n, d):
    return lib().orc_rhu(n, d)


def rsh_r(a, k):
    return lib().orc_rsh_r(a, k)


def rescale(a, M, e):
    return lib().orc_rescale(a, M, e)


def quantize_multiplier(s):
    M, e = C.c_int32(), C.c_int()
    rc = lib().orc_quantize_multiplier(s, C.byref(M), C.byref(e))
    if rc != OK:
        raise OracleError(rc, "quantize_multiplier")
    return M.value, e.value


def isqrt(v):
    return lib().orc_isqrt(v)


def expneg(y):
    return lib().orc_expneg(y)


def int_sigmoid(x, m):
    return lib().orc_int_sigmoid(x, m)


def int_tanh(x, m):
    return lib().orc_int_tanh(x, m)


def int_layernorm(q, qL, qb, M_ln, e_ln):
    q = np.ascontiguousarray(q, dtype=np.int16)
    qL = np.ascontiguousarray(qL, dtype=np.int16)
    qb = np.ascontiguousarray(qb, dtype=np.int32)
    out = np.empty_like(q)
    rc = lib().orc_int_layernorm(q.ctypes.data, q.size, qL.ctypes.data, qb.ctypes.data, M_ln, e_ln,
                                 out.ctypes.data)
    if rc != OK:
        raise OracleError(rc, "int_layernorm")
    return out


def max_threads():
    return lib().orc_max_threads()


# ---------------------------------------------------------------- marshalling
def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _marshal(layers):
    """LayerSpec-like objects -> (ctypes array, keep-alive list)."""
    arr = (_LayerParams * len(layers))()
    keep = []

    def ptr(a):
        if a is None:
            return _fp()
        a = _f32(a)
        keep.append(a)
        return a.ctypes.data_as(_fp)

    for p, s in zip(arr, layers):
        p.input_size, p.num_cells, p.output_size = s.input_size, s.num_cells, s.output_size
        p.flags = s.flags
        for g in range(4):
            p.W[g], p.R[g], p.b[g], p.Lw[g] = ptr(s.W[g]), ptr(s.R[g]), ptr(s.b[g]), ptr(s.Lw[g])
        for j in range(3):
            p.P[j] = ptr(s.P[j])
        p.Wproj, p.bproj = ptr(s.Wproj), ptr(s.bproj)
        p.x_min, p.x_max, p.h_min, p.h_max = s.x_min, s.x_max, s.h_min, s.h_max
        p.m_min, p.m_max, p.c_absmax = s.m_min, s.m_max, s.c_absmax
        for g in range(4):
            p.g_absmax[g] = s.g_absmax[g]
    return arr, keep


def _np_from(ptr, shape, dtype):
    n = int(np.prod(shape))
    return np.ctypeslib.as_array(ptr, shape=(n,)).astype(dtype).reshape(shape).copy()


class OracleModel:
    def __init__(self, handle, num_layers):
        self._h = handle
        self.num_layers = num_layers

    def __del__(self):
        if getattr(self, "_h", None):
            lib().orc_destroy(self._h)
            self._h = None

    def layer(self, l):
        """Every quantized tensor, zero point, scale and (M, e) pair of layer l."""
        q = lib().orc_get_layer(self._h, l).contents
        N, I, H = q.N, q.I, q.H
        proj = bool(q.flags & PROJECTION)
        d = {k: getattr(q, k) for k in ("I", "N", "H", "G", "flags", "m_c", "zp_x", "zp_h", "zp_m",
                                        "s_x", "s_h", "s_m", "s_c", "s_Wp", "Mm", "em", "Mp", "ep")}
        for k in ("s_W", "s_R", "s_P", "s_L", "s_g", "Mx", "ex", "Mh", "eh", "Mc", "ec", "Mln", "eln"):
            d[k] = list(getattr(q, k))
        d["Wq"] = _np_from(q.Wq, (4, N, I), np.int8)
        d["Rq"] = _np_from(q.Rq, (4, N, H), np.int8)
        d["qb"] = _np_from(q.qb, (4, N), np.int32)
        d["Pq"] = _np_from(q.Pq, (3, N), np.int16)
        d["Lq"] = _np_from(q.Lq, (4, N), np.int16)
        d["bx_fold"] = _np_from(q.bx_fold, (4, N), np.int32)
        d["bh_fold"] = _np_from(q.bh_fold, (4, N), np.int32)
        if proj:
            d["Wpq"] = _np_from(q.Wpq, (H, N), np.int8)
            d["qbp"] = _np_from(q.qbp, (H,), np.int32)
            d["bp_fold"] = _np_from(q.bp_fold, (H,), np.int32)
        return d

    def dims(self):
        out = []
        for l in range(self.num_layers):
            q = lib().orc_get_layer(self._h, l).contents
            out.append((q.I, q.N, q.H))
        return out


def prepare(layers):
    arr, keep = _marshal(layers)
    h = C.c_void_p()
    rc = lib().orc_prepare(arr, len(layers), C.byref(h))
    del keep
    if rc != OK:
        raise OracleError(rc, "prepare")
    return OracleModel(h, len(layers))


def quantize_input(x, s_x, zp_x):
    """Float features -> int8 with the first layer's (s_x, zp_x) (Sec. 3.2.4):
    q = clamp(floor(v / s + 1/2) + zp, -128, 127), in double."""
    v = np.floor(np.asarray(x, dtype=np.float64) / s_x + 0.5) + zp_x
    return np.clip(v, -128, 127).astype(np.int8)


_TRACE_FIELDS = ("tx", "th", "g", "ln", "act", "c", "m", "h")


def forward(model, xq, h_state=None, c_state=None, trace_layer=None, unfolded=False,
            threads=None, reverse=False):
    """xq int8 [T,B,I0] -> y int8 [T,B,H_last].  States (flat arrays, layers
    concatenated) are updated in place when given.  With trace_layer, also
    returns a dict of that layer's per-(t,b) integer tensors.

    reverse: the backward direction of a bidirectional layer (Sec. 7) -- the
    same recursion over the time-reversed sequence, every per-step tensor
    stored back at its position in time.  By definition: flip, run, flip."""
    if reverse:
        out = forward(model, np.ascontiguousarray(np.asarray(xq)[::-1]), h_state, c_state, trace_layer,
                      unfolded, threads)
        if trace_layer is None:
            return np.ascontiguousarray(out[::-1])
        y, bufs = out
        return np.ascontiguousarray(y[::-1]), {k: np.ascontiguousarray(v[::-1]) for k, v in bufs.items()}
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    T, B, I0 = xq.shape
    dims = model.dims()
    assert I0 == dims[0][0]
    y = np.zeros((T, B, dims[-1][2]), dtype=np.int8)
    tr = None
    bufs = {}
    if trace_layer is not None:
        I, N, H = dims[trace_layer]
        tr = _Trace()
        tr.layer = trace_layer
        for f in _TRACE_FIELDS:
            shape = {"c": (T, B, N), "m": (T, B, N), "h": (T, B, H)}.get(f, (T, B, 4, N))
            bufs[f] = np.zeros(shape, dtype=np.int8 if f in ("m", "h") else np.int16)
            setattr(tr, f, bufs[f].ctypes.data)
    if h_state is not None:
        assert h_state.dtype == np.int8 and h_state.flags.c_contiguous
        assert h_state.size == sum(B * d[2] for d in dims)
    if c_state is not None:
        assert c_state.dtype == np.int16 and c_state.flags.c_contiguous
        assert c_state.size == sum(B * d[1] for d in dims)
    rc = lib().orc_forward(model._h, xq.ctypes.data, T, B, y.ctypes.data,
                           h_state.ctypes.data if h_state is not None else None,
                           c_state.ctypes.data if c_state is not None else None,
                           C.byref(tr) if tr is not None else None, int(unfolded),
                           threads or max_threads())
    if rc != OK:
        raise OracleError(rc, "forward")
    return (y, bufs) if trace_layer is not None else y


def float_forward(layers, x, threads=None):
    """Double-precision LSTM of Sec. 2 over x float32 [T,B,I0].
    Returns (y float64 [T,B,H_last], per-layer statistics as dicts)."""
    x = _f32(x)
    T, B, _ = x.shape
    arr, keep = _marshal(layers)
    y = np.zeros((T, B, layers[-1].output_size), dtype=np.float64)
    st = (_FloatStats * len(layers))()
    rc = lib().orc_float_forward(arr, len(layers), x.ctypes.data, T, B, y.ctypes.data, st,
                                 threads or max_threads())
    del keep
    if rc != OK:
        raise OracleError(rc, "float_forward")
    stats = []
    for s in st:
        d = {k: getattr(s, k) for k in ("x_min", "x_max", "h_min", "h_max", "m_min", "m_max",
                                        "c_absmax")}
        d["g_absmax"] = list(s.g_absmax)
        stats.append(d)
    return y, stats


def apply_stats(layers, stats):
    """Copies calibration statistics into the layer specs (in place)."""
    for s, d in zip(layers, stats):
        s.x_min, s.x_max, s.h_min, s.h_max = d["x_min"], d["x_max"], d["h_min"], d["h_max"]
        s.m_min, s.m_max, s.c_absmax = d["m_min"], d["m_max"], d["c_absmax"]
        s.g_absmax = list(d["g_absmax"])
    return layers
