"""ctypes binding of the CPU oracle's integer SRU (sru_int_oracle.c, in liblstm_int_oracle.so).

TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT.  Only tests may import this
module; the HIP library and its Python binding never do, and this module
never imports them.  The recipe (Sec. 7 of arXiv 2101.05453 names the SRU and
gives none) is stated in sru_int_oracle.h.
"""
import ctypes as C

import numpy as np

from . import OK, OracleError, lib as _base_lib

_fp = C.POINTER(C.c_float)


class _SruParams(C.Structure):
    _fields_ = [
        ("input_size", C.c_int32), ("num_cells", C.c_int32),
        ("W", _fp * 4), ("v", _fp * 2), ("b", _fp * 2),
        ("x_min", C.c_float), ("x_max", C.c_float), ("c_absmax", C.c_float),
        ("h_min", C.c_float), ("h_max", C.c_float),
    ]


class _SruQuant(C.Structure):
    _fields_ = [
        ("I", C.c_int32), ("N", C.c_int32), ("G", C.c_int32),
        ("zp_x", C.c_int32), ("zp_h", C.c_int32), ("m_c", C.c_int32),
        ("s_x", C.c_double), ("s_h", C.c_double), ("s_W", C.c_double * 4), ("s_v", C.c_double * 2),
        ("Mx", C.c_int32 * 4), ("ex", C.c_int32 * 4), ("Mv", C.c_int32 * 2), ("ev", C.c_int32 * 2),
        ("Ms", C.c_int32), ("es", C.c_int32), ("Mh", C.c_int32), ("eh", C.c_int32),
        ("Wq", C.POINTER(C.c_int8)), ("vq", C.POINTER(C.c_int16)),
        ("bq", C.POINTER(C.c_int32)), ("b_fold", C.POINTER(C.c_int32)),
    ]


class _SruTrace(C.Structure):
    _fields_ = [("layer", C.c_int32)] + [(n, C.c_void_p) for n in ("tx", "tv", "act", "c", "h16", "y")]


class _SruStats(C.Structure):
    _fields_ = [("c_absmax", C.c_double), ("h_min", C.c_double), ("h_max", C.c_double)]


_ready = False


def lib():
    global _ready
    L = _base_lib()
    if not _ready:
        L.orc_sru_prepare.restype = C.c_int
        L.orc_sru_prepare.argtypes = [C.POINTER(_SruParams), C.c_int32, C.POINTER(C.c_void_p)]
        L.orc_sru_destroy.restype = None
        L.orc_sru_destroy.argtypes = [C.c_void_p]
        L.orc_sru_get_layer.restype = C.POINTER(_SruQuant)
        L.orc_sru_get_layer.argtypes = [C.c_void_p, C.c_int32]
        L.orc_sru_forward.restype = C.c_int
        L.orc_sru_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                      C.POINTER(_SruTrace), C.c_int, C.c_int]
        L.orc_sru_float_forward.restype = C.c_int
        L.orc_sru_float_forward.argtypes = [C.POINTER(_SruParams), C.c_int32, C.c_void_p, C.c_int32, C.c_int32,
                                            C.c_void_p, C.POINTER(_SruStats), C.c_int]
        _ready = True
    return L


def _marshal(layers):
    arr = (_SruParams * len(layers))()
    keep = []

    def ptr(a):
        if a is None:
            return _fp()
        a = np.ascontiguousarray(a, dtype=np.float32)
        keep.append(a)
        return a.ctypes.data_as(_fp)

    for p, s in zip(arr, layers):
        p.input_size, p.num_cells = s.input_size, s.num_cells
        for g in range(4):
            p.W[g] = ptr(s.W[g])
        for j in range(2):
            p.v[j], p.b[j] = ptr(s.v[j]), ptr(s.b[j])
        p.x_min, p.x_max, p.c_absmax, p.h_min, p.h_max = s.x_min, s.x_max, s.c_absmax, s.h_min, s.h_max
    return arr, keep


TRACE_FIELDS = {"tx": (np.int16, 4), "tv": (np.int16, 2), "act": (np.int16, 2), "c": (np.int16, 0),
                "h16": (np.int16, 0), "y": (np.int8, 0)}


class SruModel:
    """Integer SRU prepared by the oracle."""

    def __init__(self, layers):
        self._h = C.c_void_p()
        arr, keep = _marshal(layers)
        rc = lib().orc_sru_prepare(arr, len(layers), C.byref(self._h))
        if rc != OK:
            raise OracleError(rc, "sru_prepare")
        self.num_layers = len(layers)

    def __del__(self):
        if getattr(self, "_h", None) and self._h.value:
            lib().orc_sru_destroy(self._h)
            self._h = C.c_void_p()

    def get_quant(self, layer):
        q = lib().orc_sru_get_layer(self._h, layer).contents
        I, N, G = q.I, q.N, q.G
        out = {k: getattr(q, k) for k in ("I", "N", "G", "zp_x", "zp_h", "m_c", "s_x", "s_h", "Ms", "es", "Mh", "eh")}
        for k in ("s_W", "s_v", "Mx", "ex", "Mv", "ev"):
            out[k] = list(getattr(q, k))
        out["Wq"] = np.ctypeslib.as_array(q.Wq, shape=(G, N, I)).copy()
        out["vq"] = np.ctypeslib.as_array(q.vq, shape=(2, N)).copy()
        for k in ("bq", "b_fold"):
            out[k] = np.ctypeslib.as_array(getattr(q, k), shape=(G, N)).copy()
        return out

    def forward(self, xq, c_state=None, trace_layer=None, unfolded=False, threads=1):
        """xq int8 [T,B,I0] -> (y int8 [T,B,N_last], trace dict or None); c_state (int16, layers
        concatenated) is updated in place when given."""
        xq = np.ascontiguousarray(xq, dtype=np.int8)
        T, B, _ = xq.shape
        N_last = lib().orc_sru_get_layer(self._h, self.num_layers - 1).contents.N
        y = np.zeros((T, B, N_last), dtype=np.int8)
        tr, trp = None, None
        if trace_layer is not None:
            N = lib().orc_sru_get_layer(self._h, trace_layer).contents.N
            tr = {k: np.zeros((T, B, g, N) if g else (T, B, N), dtype=dt) for k, (dt, g) in TRACE_FIELDS.items()}
            trp = _SruTrace(layer=trace_layer, **{k: v.ctypes.data for k, v in tr.items()})
        if c_state is not None:
            assert c_state.dtype == np.int16 and c_state.flags["C_CONTIGUOUS"]
        rc = lib().orc_sru_forward(self._h, xq.ctypes.data, T, B, y.ctypes.data,
                                   c_state.ctypes.data if c_state is not None else None,
                                   C.byref(trp) if trp is not None else None, int(unfolded), threads)
        if rc != OK:
            raise OracleError(rc, "sru_forward")
        return y, tr


def float_forward(layers, x, threads=1):
    """The float SRU in double: x float32 [T,B,I0] -> (y float64 [T,B,N_last], per-layer statistics
    [{c_absmax, h_min, h_max}])."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    T, B, _ = x.shape
    arr, keep = _marshal(layers)
    y = np.zeros((T, B, layers[-1].num_cells), dtype=np.float64)
    st = (_SruStats * len(layers))()
    rc = lib().orc_sru_float_forward(arr, len(layers), x.ctypes.data, T, B, y.ctypes.data, st, threads)
    if rc != OK:
        raise OracleError(rc, "sru_float_forward")
    return y, [{"c_absmax": s.c_absmax, "h_min": s.h_min, "h_max": s.h_max} for s in st]


def calibrate(layers, x, threads=1):
    """Sets c_absmax, h_min, h_max of every layer from a float run over x (Sec. 4); returns the float output."""
    y, stats = float_forward(layers, x, threads)
    for s, st in zip(layers, stats):
        s.c_absmax, s.h_min, s.h_max = st["c_absmax"], st["h_min"], st["h_max"]
    return y
