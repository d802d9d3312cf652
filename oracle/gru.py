"""ctypes binding of the CPU oracle's integer GRU (gru_int_oracle.c, in liblstm_int_oracle.so).

TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT.  Only tests may import this
module; the HIP library and its Python binding never do, and this module
never imports them.  The recipe (Sec. 7 of arXiv 2101.05453 names the GRU and
gives none) is stated in gru_int_oracle.h.
"""
import ctypes as C

import numpy as np

from . import OK, OracleError, lib as _base_lib

_fp = C.POINTER(C.c_float)


class _GruParams(C.Structure):
    _fields_ = [
        ("input_size", C.c_int32), ("num_cells", C.c_int32),
        ("W", _fp * 3), ("R", _fp * 3), ("bx", _fp * 3), ("bh", _fp * 3),
        ("x_min", C.c_float), ("x_max", C.c_float),
    ]


class _GruQuant(C.Structure):
    _fields_ = [
        ("I", C.c_int32), ("N", C.c_int32), ("zp_x", C.c_int32),
        ("s_x", C.c_double), ("s_W", C.c_double * 3), ("s_R", C.c_double * 3),
        ("Mx", C.c_int32 * 3), ("ex", C.c_int32 * 3), ("Mh", C.c_int32 * 3), ("eh", C.c_int32 * 3),
        ("Wq", C.POINTER(C.c_int8)), ("Rq", C.POINTER(C.c_int8)),
        ("bxq", C.POINTER(C.c_int32)), ("bhq", C.POINTER(C.c_int32)), ("bx_fold", C.POINTER(C.c_int32)),
    ]


class _GruTrace(C.Structure):
    _fields_ = [("layer", C.c_int32)] + [(n, C.c_void_p) for n in ("tx", "th", "act", "h16", "h8")]


_ready = False


def lib():
    global _ready
    L = _base_lib()
    if not _ready:
        L.orc_gru_prepare.restype = C.c_int
        L.orc_gru_prepare.argtypes = [C.POINTER(_GruParams), C.c_int32, C.POINTER(C.c_void_p)]
        L.orc_gru_destroy.restype = None
        L.orc_gru_destroy.argtypes = [C.c_void_p]
        L.orc_gru_get_layer.restype = C.POINTER(_GruQuant)
        L.orc_gru_get_layer.argtypes = [C.c_void_p, C.c_int32]
        L.orc_gru_forward.restype = C.c_int
        L.orc_gru_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                      C.POINTER(_GruTrace), C.c_int, C.c_int]
        L.orc_gru_float_forward.restype = C.c_int
        L.orc_gru_float_forward.argtypes = [C.POINTER(_GruParams), C.c_int32, C.c_void_p, C.c_int32, C.c_int32,
                                            C.c_void_p, C.c_int]
        _ready = True
    return L


def _marshal(layers):
    arr = (_GruParams * len(layers))()
    keep = []

    def ptr(a):
        a = np.ascontiguousarray(a, dtype=np.float32)
        keep.append(a)
        return a.ctypes.data_as(_fp)

    for p, s in zip(arr, layers):
        p.input_size, p.num_cells = s.input_size, s.num_cells
        for g in range(3):
            p.W[g], p.R[g], p.bx[g], p.bh[g] = ptr(s.W[g]), ptr(s.R[g]), ptr(s.bx[g]), ptr(s.bh[g])
        p.x_min, p.x_max = s.x_min, s.x_max
    return arr, keep


TRACE_FIELDS = {"tx": (np.int16, 3), "th": (np.int16, 3), "act": (np.int16, 3), "h16": (np.int16, 0), "h8": (np.int8, 0)}


class GruModel:
    """Integer GRU prepared by the oracle."""

    def __init__(self, layers):
        self._h = C.c_void_p()
        arr, keep = _marshal(layers)
        rc = lib().orc_gru_prepare(arr, len(layers), C.byref(self._h))
        if rc != OK:
            raise OracleError(rc, "gru_prepare")
        self.num_layers = len(layers)

    def __del__(self):
        if getattr(self, "_h", None) and self._h.value:
            lib().orc_gru_destroy(self._h)
            self._h = C.c_void_p()

    def get_quant(self, layer):
        q = lib().orc_gru_get_layer(self._h, layer).contents
        I, N = q.I, q.N
        out = {k: getattr(q, k) for k in ("I", "N", "zp_x", "s_x")}
        for k in ("s_W", "s_R", "Mx", "ex", "Mh", "eh"):
            out[k] = list(getattr(q, k))
        out["Wq"] = np.ctypeslib.as_array(q.Wq, shape=(3, N, I)).copy()
        out["Rq"] = np.ctypeslib.as_array(q.Rq, shape=(3, N, N)).copy()
        for k in ("bxq", "bhq", "bx_fold"):
            out[k] = np.ctypeslib.as_array(getattr(q, k), shape=(3, N)).copy()
        return out

    def forward(self, xq, h_state=None, trace_layer=None, unfolded=False, threads=1):
        """xq int8 [T,B,I0] -> (y int8 [T,B,N_last], trace dict or None); h_state (int16, layers
        concatenated) is updated in place when given."""
        xq = np.ascontiguousarray(xq, dtype=np.int8)
        T, B, _ = xq.shape
        N_last = lib().orc_gru_get_layer(self._h, self.num_layers - 1).contents.N
        y = np.zeros((T, B, N_last), dtype=np.int8)
        tr, trp = None, None
        if trace_layer is not None:
            N = lib().orc_gru_get_layer(self._h, trace_layer).contents.N
            tr = {k: np.zeros((T, B, g, N) if g else (T, B, N), dtype=dt) for k, (dt, g) in TRACE_FIELDS.items()}
            trp = _GruTrace(layer=trace_layer, **{k: v.ctypes.data for k, v in tr.items()})
        if h_state is not None:
            assert h_state.dtype == np.int16 and h_state.flags["C_CONTIGUOUS"]
        rc = lib().orc_gru_forward(self._h, xq.ctypes.data, T, B, y.ctypes.data,
                                   h_state.ctypes.data if h_state is not None else None,
                                   C.byref(trp) if trp is not None else None, int(unfolded), threads)
        if rc != OK:
            raise OracleError(rc, "gru_forward")
        return y, tr


def float_forward(layers, x, threads=1):
    """The float GRU in double: x float32 [T,B,I0] -> y float64 [T,B,N_last]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    T, B, _ = x.shape
    arr, keep = _marshal(layers)
    y = np.zeros((T, B, layers[-1].num_cells), dtype=np.float64)
    rc = lib().orc_gru_float_forward(arr, len(layers), x.ctypes.data, T, B, y.ctypes.data, threads)
    if rc != OK:
        raise OracleError(rc, "gru_float_forward")
    return y
