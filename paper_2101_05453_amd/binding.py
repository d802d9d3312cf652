"""ctypes binding of liblstm_int.so: the same entry points as include/lstm_int.h.

Argument marshalling only -- every step of the path runs in the library's
kernels.  PyTorch supplies device memory and streams.  There is no fallback:
if the library is missing or the call fails, an exception is raised.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblstm_int.so")

CIFG, PEEPHOLE, LAYER_NORM, PROJECTION = 1, 2, 4, 8
OK = 0
E_INVALID_ARG, E_UNSUPPORTED, E_BAD_RANGE, E_OUT_OF_MEMORY, E_DEVICE, E_WORKSPACE = -1, -2, -3, -4, -5, -6
K_INPUT_GEMM, K_RECURRENT, K_CELL, K_PROJECTION, K_OTHER, K_COUNT = 0, 1, 2, 3, 4, 5
KERNEL_CLASSES = ("input_gemm", "recurrent", "cell", "projection", "other")
STATIC_WORKSPACE_BYTES = 32 << 20  # LSTM_INT_STATIC_WORKSPACE_BYTES

_fp = C.POINTER(C.c_float)


class LayerParams(C.Structure):
    """lstm_int_layer_params"""
    _fields_ = [
        ("input_size", C.c_int32), ("num_cells", C.c_int32), ("output_size", C.c_int32),
        ("flags", C.c_uint32),
        ("W", _fp * 4), ("R", _fp * 4), ("b", _fp * 4), ("P", _fp * 3), ("Lw", _fp * 4),
        ("Wproj", _fp), ("bproj", _fp),
        ("x_min", C.c_float), ("x_max", C.c_float), ("h_min", C.c_float), ("h_max", C.c_float),
        ("m_min", C.c_float), ("m_max", C.c_float), ("c_absmax", C.c_float),
        ("g_absmax", C.c_float * 4),
    ]


class LayerStats(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("x_min", "x_max", "h_min", "h_max", "m_min", "m_max", "c_absmax")] + [
        ("g_absmax", C.c_double * 4)]


class LayerQuant(C.Structure):
    """lstm_int_layer_quant"""
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


class Trace(C.Structure):
    """lstm_int_trace"""
    _fields_ = [("layer", C.c_int32)] + [
        (n, C.c_void_p) for n in ("tx", "th", "g", "ln", "act", "c", "m", "h")
    ]


TRACE_FIELDS = ("tx", "th", "g", "ln", "act", "c", "m", "h")

_lib = None


class LstmIntError(RuntimeError):
    def __init__(self, code, what):
        msg = lib().lstm_int_strerror(code).decode() if _lib is not None else "?"
        super().__init__(f"{what}: {msg} ({code})")
        self.code = code


def lib():
    """Loads liblstm_int.so (built by paper_2101_05453_amd.build); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run python -m paper_2101_05453_amd.build")
        try:
            # torch first: it brings a HIP runtime of its own, and the library has to meet that one in the process
            # (loaded before torch, the library pulled in the system's runtime and every call on a torch tensor
            # then failed with a device error)
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        L.lstm_int_prepare.restype = C.c_int
        L.lstm_int_prepare.argtypes = [C.POINTER(LayerParams), C.c_int32, C.c_int32,
                                       C.POINTER(C.c_void_p)]
        L.lstm_int_get_quant.restype = C.c_int
        L.lstm_int_get_quant.argtypes = [C.c_void_p, C.c_int32, C.POINTER(LayerQuant)]
        L.lstm_int_quantize_input.restype = C.c_int
        L.lstm_int_quantize_input.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        L.lstm_int_workspace_bytes.restype = C.c_size_t
        L.lstm_int_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        L.lstm_int_forward.restype = C.c_int
        L.lstm_int_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p,
                                       C.POINTER(Trace)]
        L.lstm_int_forward_static.restype = C.c_int
        L.lstm_int_forward_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p]
        L.lstm_int_bidirectional_workspace_bytes.restype = C.c_size_t
        L.lstm_int_bidirectional_workspace_bytes.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32]
        L.lstm_int_forward_bidirectional.restype = C.c_int
        L.lstm_int_forward_bidirectional.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                     C.c_void_p, C.c_size_t, C.c_void_p]
        L.lstm_int_set_option.restype = C.c_int
        L.lstm_int_set_option.argtypes = [C.c_void_p, C.c_char_p, C.c_int64]
        L.lstm_int_device_status.restype = C.c_int
        L.lstm_int_device_status.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
        L.lstm_int_sparse_layers.restype = C.c_int
        L.lstm_int_sparse_layers.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
        L.lstm_int_phase_ticks.restype = C.c_int
        L.lstm_int_phase_ticks.argtypes = [C.c_void_p, C.POINTER(C.c_int64)]
        L.lstm_int_profile_begin.restype = C.c_int
        L.lstm_int_profile_begin.argtypes = [C.c_void_p]
        L.lstm_int_profile_end.restype = C.c_int
        L.lstm_int_profile_end.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_double)]
        L.lstm_int_calibrate.restype = C.c_int
        L.lstm_int_calibrate.argtypes = [C.POINTER(LayerParams), C.c_int32, C.c_int32, C.c_void_p, C.c_int32,
                                         C.c_int32, C.c_void_p, C.POINTER(LayerStats), C.c_void_p]
        L.lstm_int_lds_probe.restype = C.c_int
        L.lstm_int_lds_probe.argtypes = [C.c_int32] * 5
        L.lstm_int_mfma_store_ceiling.restype = C.c_int
        L.lstm_int_mfma_store_ceiling.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_double),
                                                  C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.lstm_int_destroy.restype = None
        L.lstm_int_destroy.argtypes = [C.c_void_p]
        L.lstm_int_strerror.restype = C.c_char_p
        L.lstm_int_strerror.argtypes = [C.c_int]
        _lib = L
    return _lib


def _check(rc, what):
    if rc != OK:
        raise LstmIntError(rc, what)


def marshal_layers(layers):
    """LayerSpec-like objects -> (ctypes array of lstm_int_layer_params, keep-alive list)."""
    arr = (LayerParams * len(layers))()
    keep = []

    def ptr(a):
        if a is None:
            return _fp()
        a = np.ascontiguousarray(a, dtype=np.float32)
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


def _view(ptr, shape, dtype):
    if not ptr:
        return None
    n = int(np.prod(shape))
    return np.ctypeslib.as_array(ptr, shape=(n,)).astype(dtype).reshape(shape).copy()


class Model:
    """Owns one lstm_int_model."""

    def __init__(self, handle, num_layers, device):
        self._h = handle
        self.num_layers = num_layers
        self.device = device

    def __del__(self):
        self.destroy()

    def destroy(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.lstm_int_destroy(self._h)
        self._h = None

    # lstm_int_get_quant
    def get_quant(self, layer):
        q = LayerQuant()
        _check(lib().lstm_int_get_quant(self._h, layer, C.byref(q)), "lstm_int_get_quant")
        N, I, H = q.N, q.I, q.H
        d = {k: getattr(q, k) for k in ("I", "N", "H", "G", "flags", "m_c", "zp_x", "zp_h", "zp_m",
                                        "s_x", "s_h", "s_m", "s_c", "s_Wp", "Mm", "em", "Mp", "ep")}
        for k in ("s_W", "s_R", "s_P", "s_L", "s_g", "Mx", "ex", "Mh", "eh", "Mc", "ec", "Mln", "eln"):
            d[k] = list(getattr(q, k))
        d["Wq"] = _view(q.Wq, (4, N, I), np.int8)
        d["Rq"] = _view(q.Rq, (4, N, H), np.int8)
        d["qb"] = _view(q.qb, (4, N), np.int32)
        d["Pq"] = _view(q.Pq, (3, N), np.int16)
        d["Lq"] = _view(q.Lq, (4, N), np.int16)
        d["bx_fold"] = _view(q.bx_fold, (4, N), np.int32)
        d["bh_fold"] = _view(q.bh_fold, (4, N), np.int32)
        if q.flags & PROJECTION:
            d["Wpq"] = _view(q.Wpq, (H, N), np.int8)
            d["qbp"] = _view(q.qbp, (H,), np.int32)
            d["bp_fold"] = _view(q.bp_fold, (H,), np.int32)
        return d

    def dims(self):
        if getattr(self, "_dims", None):
            return self._dims
        out = []
        for l in range(self.num_layers):
            q = LayerQuant()
            _check(lib().lstm_int_get_quant(self._h, l, C.byref(q)), "lstm_int_get_quant")
            out.append((q.I, q.N, q.H))
        self._dims = out
        return out

    # lstm_int_quantize_input on a torch device tensor
    def quantize_input(self, x, out=None):
        """x: float32 CUDA tensor of features (any shape) -> int8 CUDA tensor of
        the same shape, the codes layer 0 reads.  Asynchronous on torch's current
        stream."""
        import torch

        assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
        if out is None:
            out = torch.empty(x.shape, dtype=torch.int8, device=x.device)
        assert out.is_cuda and out.dtype == torch.int8 and out.is_contiguous() and out.numel() == x.numel()
        stream = torch.cuda.current_stream(x.device).cuda_stream
        _check(lib().lstm_int_quantize_input(self._h, x.data_ptr(), x.numel(), out.data_ptr(), stream),
               "lstm_int_quantize_input")
        return out

    # lstm_int_workspace_bytes
    def workspace_bytes(self, T, B):
        return lib().lstm_int_workspace_bytes(self._h, T, B)

    # lstm_int_set_option
    def set_option(self, key, value):
        _check(lib().lstm_int_set_option(self._h, key.encode(), value), "lstm_int_set_option")

    # lstm_int_sparse_layers
    def sparse_layers(self):
        v = C.c_int32(0)
        _check(lib().lstm_int_sparse_layers(self._h, C.byref(v)), "lstm_int_sparse_layers")
        return v.value

    # lstm_int_device_status
    def device_status(self):
        v = C.c_int32()
        _check(lib().lstm_int_device_status(self._h, C.byref(v)), "lstm_int_device_status")
        return v.value

    # lstm_int_phase_ticks
    def phase_ticks(self):
        t = (C.c_int64 * 16)()
        _check(lib().lstm_int_phase_ticks(self._h, t), "lstm_int_phase_ticks")
        return list(t)

    # lstm_int_profile_begin / lstm_int_profile_end
    def profile_begin(self):
        _check(lib().lstm_int_profile_begin(self._h), "lstm_int_profile_begin")

    def profile_end(self):
        n = (C.c_int64 * K_COUNT)()
        ms = (C.c_double * K_COUNT)()
        _check(lib().lstm_int_profile_end(self._h, n, ms), "lstm_int_profile_end")
        return {k: {"launches": int(n[i]), "total_ms": float(ms[i])}
                for i, k in enumerate(KERNEL_CLASSES)}

    # lstm_int_forward, raw pointers
    def forward_ptr(self, x_ptr, T, B, y_ptr, h_ptr, c_ptr, ws_ptr, ws_bytes, stream_ptr, trace=None):
        _check(lib().lstm_int_forward(self._h, x_ptr, T, B, y_ptr, h_ptr, c_ptr, ws_ptr, ws_bytes,
                                      stream_ptr, C.byref(trace) if trace is not None else None),
               "lstm_int_forward")

    # lstm_int_forward_static on torch device tensors (y must be given: the call allocates nothing)
    def forward_static(self, x, y, h_state=None, c_state=None):
        import torch

        assert x.is_cuda and x.dtype == torch.int8 and x.is_contiguous()
        assert y.is_cuda and y.dtype == torch.int8 and y.is_contiguous()
        T, B, _ = x.shape
        assert tuple(y.shape) == (T, B, self.dims()[-1][2])
        stream = torch.cuda.current_stream(x.device).cuda_stream
        _check(lib().lstm_int_forward_static(self._h, x.data_ptr(), T, B, y.data_ptr(),
                                             h_state.data_ptr() if h_state is not None else None,
                                             c_state.data_ptr() if c_state is not None else None, stream),
               "lstm_int_forward_static")
        return y

    # lstm_int_forward on torch device tensors
    def forward(self, x, y=None, h_state=None, c_state=None, workspace=None, trace_layer=None):
        """x: int8 CUDA tensor [T,B,I0].  Returns y (int8 [T,B,H_last]); with
        trace_layer also a dict of that layer's intermediate tensors.  The call
        is asynchronous on torch's current stream."""
        import torch

        assert x.is_cuda and x.dtype == torch.int8 and x.is_contiguous()
        T, B, _ = x.shape
        dims = self.dims()
        if y is None:
            y = torch.empty((T, B, dims[-1][2]), dtype=torch.int8, device=x.device)
        need = self.workspace_bytes(T, B)
        if workspace is None:
            workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
        tr, bufs = None, {}
        if trace_layer is not None:
            I, N, H = dims[trace_layer]
            tr = Trace()
            tr.layer = trace_layer
            for f in TRACE_FIELDS:
                shape = {"c": (T, B, N), "m": (T, B, N), "h": (T, B, H)}.get(f, (T, B, 4, N))
                dt = torch.int8 if f in ("m", "h") else torch.int16
                bufs[f] = torch.zeros(shape, dtype=dt, device=x.device)
                setattr(tr, f, bufs[f].data_ptr())
        stream = torch.cuda.current_stream(x.device).cuda_stream
        self.forward_ptr(x.data_ptr(), T, B, y.data_ptr(),
                         h_state.data_ptr() if h_state is not None else None,
                         c_state.data_ptr() if c_state is not None else None,
                         workspace.data_ptr(), workspace.numel(), stream, tr)
        return (y, bufs) if trace_layer is not None else y


# lstm_int_prepare
def prepare(layers, device=0):
    """layers: LayerSpec-like objects with calibration statistics filled in.
    device = -1 builds a host-only model (no GPU needed)."""
    arr, keep = marshal_layers(layers)
    h = C.c_void_p()
    rc = lib().lstm_int_prepare(arr, len(layers), device, C.byref(h))
    del keep
    _check(rc, "lstm_int_prepare")
    return Model(h, len(layers), device)


# lstm_int_bidirectional_workspace_bytes
def bidirectional_workspace_bytes(fwd, bwd, T, B):
    return lib().lstm_int_bidirectional_workspace_bytes(fwd._h, bwd._h, T, B)


# lstm_int_forward_bidirectional on torch device tensors
def forward_bidirectional(fwd, bwd, x, y=None, state_fwd=(None, None), state_bwd=(None, None), workspace=None):
    """fwd, bwd: Models on the same device, bwd with option "reverse" = 1.  x: int8 CUDA tensor [T,B,I0].
    Returns y int8 [T,B,H_fwd + H_bwd].  Asynchronous on torch's current stream."""
    import torch

    assert x.is_cuda and x.dtype == torch.int8 and x.is_contiguous()
    T, B, _ = x.shape
    Hf, Hb = fwd.dims()[-1][2], bwd.dims()[-1][2]
    if y is None:
        y = torch.empty((T, B, Hf + Hb), dtype=torch.int8, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(bidirectional_workspace_bytes(fwd, bwd, T, B), 256), dtype=torch.uint8, device=x.device)
    p = lambda t: t.data_ptr() if t is not None else None
    stream = torch.cuda.current_stream(x.device).cuda_stream
    _check(lib().lstm_int_forward_bidirectional(fwd._h, bwd._h, x.data_ptr(), T, B, y.data_ptr(), p(state_fwd[0]),
                                                p(state_fwd[1]), p(state_bwd[0]), p(state_bwd[1]), workspace.data_ptr(),
                                                workspace.numel(), stream), "lstm_int_forward_bidirectional")
    return y


# lstm_int_calibrate
def calibrate(layers, x, device=0, want_output=False, apply=True, max_rows=None):
    """Statistics of a float run on the GPU.  x: float32 CUDA tensor [T,B,I0]
    (the calibration rows; max_rows keeps only the first rows of the batch).  Returns the per-layer statistics as dicts (and the
    float output of the last layer, a float64 CUDA tensor, with want_output);
    with apply they are also written into the layer specs, ready for prepare."""
    import torch

    if max_rows is not None and x.shape[1] > max_rows:
        x = x[:, :max_rows].contiguous()
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
    T, B, _ = x.shape
    arr, keep = marshal_layers(layers)
    st = (LayerStats * len(layers))()
    y = torch.empty((T, B, layers[-1].output_size), dtype=torch.float64, device=x.device) if want_output else None
    stream = torch.cuda.current_stream(x.device).cuda_stream
    rc = lib().lstm_int_calibrate(arr, len(layers), device, x.data_ptr(), T, B, stream, st,
                                  y.data_ptr() if y is not None else None)
    del keep
    _check(rc, "lstm_int_calibrate")
    stats = []
    for spec, r in zip(layers, st):
        d = {k: getattr(r, k) for k in ("x_min", "x_max", "h_min", "h_max", "m_min", "m_max", "c_absmax")}
        d["g_absmax"] = list(r.g_absmax)
        stats.append(d)
        if apply:
            spec.x_min, spec.x_max, spec.h_min, spec.h_max = d["x_min"], d["x_max"], d["h_min"], d["h_max"]
            spec.m_min, spec.m_max, spec.c_absmax = d["m_min"], d["m_max"], d["c_absmax"]
            spec.g_absmax = list(d["g_absmax"])
    return (stats, y) if want_output else stats


# lstm_int_lds_probe
def lds_probe(map, stride_words, swizzle=0, write=False, device=0):
    """One launch of the LDS access pattern probe (see lstm_int.h); its cost is read from rocprofv3's counters."""
    _check(lib().lstm_int_lds_probe(device, map, stride_words, swizzle, int(write)), "lstm_int_lds_probe")


# lstm_int_mfma_store_ceiling
def mfma_store_ceiling(stores_per_block, blocks=4096, device=0):
    """Sustained int8 MFMA rate with `stores_per_block` KB of streaming stores per 40 MFMAs and wave."""
    t, g, c = C.c_double(), C.c_double(), C.c_double()
    _check(lib().lstm_int_mfma_store_ceiling(device, stores_per_block, blocks, C.byref(t), C.byref(g), C.byref(c)),
           "lstm_int_mfma_store_ceiling")
    return {"stores_per_block": stores_per_block, "tops": t.value, "store_gbs": g.value, "clock_ghz": c.value}


def strerror(code):
    return lib().lstm_int_strerror(code).decode()


# ---------------------------------------------------------------------------
# gru_int_* (include/gru_int.h): the integer GRU built from the same blocks
# ---------------------------------------------------------------------------
class GruLayerParams(C.Structure):
    """gru_int_layer_params"""
    _fields_ = [
        ("input_size", C.c_int32), ("num_cells", C.c_int32),
        ("W", _fp * 3), ("R", _fp * 3), ("bx", _fp * 3), ("bh", _fp * 3),
        ("x_min", C.c_float), ("x_max", C.c_float),
    ]


class GruLayerQuant(C.Structure):
    """gru_int_layer_quant"""
    _fields_ = [
        ("I", C.c_int32), ("N", C.c_int32), ("zp_x", C.c_int32),
        ("s_x", C.c_double), ("s_W", C.c_double * 3), ("s_R", C.c_double * 3),
        ("Mx", C.c_int32 * 3), ("ex", C.c_int32 * 3), ("Mh", C.c_int32 * 3), ("eh", C.c_int32 * 3),
        ("Wq", C.POINTER(C.c_int8)), ("Rq", C.POINTER(C.c_int8)),
        ("bxq", C.POINTER(C.c_int32)), ("bhq", C.POINTER(C.c_int32)), ("bx_fold", C.POINTER(C.c_int32)),
    ]


class GruTrace(C.Structure):
    """gru_int_trace"""
    _fields_ = [("layer", C.c_int32)] + [(n, C.c_void_p) for n in ("tx", "th", "act", "h16", "h8")]


GRU_TRACE_FIELDS = ("tx", "th", "act", "h16", "h8")
_gru_ready = False


def gru_lib():
    global _gru_ready
    L = lib()
    if not _gru_ready:
        L.gru_int_prepare.restype = C.c_int
        L.gru_int_prepare.argtypes = [C.POINTER(GruLayerParams), C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
        L.gru_int_get_quant.restype = C.c_int
        L.gru_int_get_quant.argtypes = [C.c_void_p, C.c_int32, C.POINTER(GruLayerQuant)]
        L.gru_int_workspace_bytes.restype = C.c_size_t
        L.gru_int_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        L.gru_int_forward.restype = C.c_int
        L.gru_int_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(GruTrace)]
        L.gru_int_set_option.restype = C.c_int
        L.gru_int_set_option.argtypes = [C.c_void_p, C.c_char_p, C.c_int64]
        L.gru_int_device_status.restype = C.c_int
        L.gru_int_device_status.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
        L.gru_int_profile_begin.restype = C.c_int
        L.gru_int_profile_begin.argtypes = [C.c_void_p]
        L.gru_int_profile_end.restype = C.c_int
        L.gru_int_profile_end.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_double)]
        L.gru_int_destroy.restype = None
        L.gru_int_destroy.argtypes = [C.c_void_p]
        _gru_ready = True
    return L


def marshal_gru_layers(layers):
    arr = (GruLayerParams * len(layers))()
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


class GruModel:
    """Owns one gru_int_model."""

    def __init__(self, handle, num_layers, device):
        self._h = handle
        self.num_layers = num_layers
        self.device = device

    def __del__(self):
        self.destroy()

    # gru_int_destroy
    def destroy(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.gru_int_destroy(self._h)
        self._h = None

    # gru_int_get_quant
    def get_quant(self, layer):
        q = GruLayerQuant()
        _check(gru_lib().gru_int_get_quant(self._h, layer, C.byref(q)), "gru_int_get_quant")
        N, I = q.N, q.I
        d = {k: getattr(q, k) for k in ("I", "N", "zp_x", "s_x")}
        for k in ("s_W", "s_R", "Mx", "ex", "Mh", "eh"):
            d[k] = list(getattr(q, k))
        d["Wq"] = _view(q.Wq, (3, N, I), np.int8)
        d["Rq"] = _view(q.Rq, (3, N, N), np.int8)
        for k in ("bxq", "bhq", "bx_fold"):
            d[k] = _view(getattr(q, k), (3, N), np.int32)
        return d

    # gru_int_workspace_bytes
    def workspace_bytes(self, T, B):
        return gru_lib().gru_int_workspace_bytes(self._h, T, B)

    # gru_int_set_option
    def set_option(self, key, value):
        _check(gru_lib().gru_int_set_option(self._h, key.encode(), value), "gru_int_set_option")

    # gru_int_device_status
    def device_status(self):
        v = C.c_int32()
        _check(gru_lib().gru_int_device_status(self._h, C.byref(v)), "gru_int_device_status")
        return v.value

    # gru_int_profile_begin / gru_int_profile_end
    def profile_begin(self):
        _check(gru_lib().gru_int_profile_begin(self._h), "gru_int_profile_begin")

    def profile_end(self):
        n = (C.c_int64 * 2)()
        ms = (C.c_double * 2)()
        _check(gru_lib().gru_int_profile_end(self._h, n, ms), "gru_int_profile_end")
        return {k: {"launches": int(n[i]), "total_ms": float(ms[i])} for i, k in enumerate(("input_gemm", "step"))}

    # gru_int_forward on torch device tensors
    def forward(self, x, y=None, h_state=None, workspace=None, trace_layer=None):
        """x: int8 CUDA tensor [T,B,I0].  Returns y (int8 [T,B,N_last]); with trace_layer also a dict of
        that layer's intermediate tensors.  Asynchronous on torch's current stream."""
        import torch

        assert x.is_cuda and x.dtype == torch.int8 and x.is_contiguous()
        T, B, _ = x.shape
        ql = GruLayerQuant()
        _check(gru_lib().gru_int_get_quant(self._h, self.num_layers - 1, C.byref(ql)), "gru_int_get_quant")
        if y is None:
            y = torch.empty((T, B, ql.N), dtype=torch.int8, device=x.device)
        if workspace is None:
            workspace = torch.empty(max(self.workspace_bytes(T, B), 256), dtype=torch.uint8, device=x.device)
        tr, bufs = None, {}
        if trace_layer is not None:
            qt = GruLayerQuant()
            _check(gru_lib().gru_int_get_quant(self._h, trace_layer, C.byref(qt)), "gru_int_get_quant")
            tr = GruTrace()
            tr.layer = trace_layer
            for f in GRU_TRACE_FIELDS:
                shape = (T, B, qt.N) if f in ("h16", "h8") else (T, B, 3, qt.N)
                bufs[f] = torch.zeros(shape, dtype=torch.int8 if f == "h8" else torch.int16, device=x.device)
                setattr(tr, f, bufs[f].data_ptr())
        if h_state is not None:
            assert h_state.is_cuda and h_state.dtype == torch.int16 and h_state.is_contiguous()
        stream = torch.cuda.current_stream(x.device).cuda_stream
        _check(gru_lib().gru_int_forward(self._h, x.data_ptr(), T, B, y.data_ptr(),
                                         h_state.data_ptr() if h_state is not None else None,
                                         workspace.data_ptr(), workspace.numel(), stream,
                                         C.byref(tr) if tr is not None else None), "gru_int_forward")
        return (y, bufs) if trace_layer is not None else y


# gru_int_prepare
def gru_prepare(layers, device=0):
    """layers: GruLayerSpec-like objects (x_min / x_max of layer 0 filled in).  device = -1 builds a
    host-only model."""
    arr, keep = marshal_gru_layers(layers)
    h = C.c_void_p()
    rc = gru_lib().gru_int_prepare(arr, len(layers), device, C.byref(h))
    del keep
    _check(rc, "gru_int_prepare")
    return GruModel(h, len(layers), device)


# ---------------------------------------------------------------------------
# sru_int_* (include/sru_int.h): the integer SRU built from the same blocks
# ---------------------------------------------------------------------------
class SruLayerParams(C.Structure):
    """sru_int_layer_params"""
    _fields_ = [
        ("input_size", C.c_int32), ("num_cells", C.c_int32),
        ("W", _fp * 4), ("v", _fp * 2), ("b", _fp * 2),
        ("x_min", C.c_float), ("x_max", C.c_float), ("c_absmax", C.c_float),
        ("h_min", C.c_float), ("h_max", C.c_float),
    ]


class SruLayerQuant(C.Structure):
    """sru_int_layer_quant"""
    _fields_ = [
        ("I", C.c_int32), ("N", C.c_int32), ("G", C.c_int32),
        ("zp_x", C.c_int32), ("zp_h", C.c_int32), ("m_c", C.c_int32),
        ("s_x", C.c_double), ("s_h", C.c_double), ("s_W", C.c_double * 4), ("s_v", C.c_double * 2),
        ("Mx", C.c_int32 * 4), ("ex", C.c_int32 * 4), ("Mv", C.c_int32 * 2), ("ev", C.c_int32 * 2),
        ("Ms", C.c_int32), ("es", C.c_int32), ("Mh", C.c_int32), ("eh", C.c_int32),
        ("Wq", C.POINTER(C.c_int8)), ("vq", C.POINTER(C.c_int16)),
        ("bq", C.POINTER(C.c_int32)), ("b_fold", C.POINTER(C.c_int32)),
    ]


SRU_TRACE_FIELDS = {"tx": 4, "tv": 2, "act": 2, "c": 0, "h16": 0, "y": 0}  # slots per (t, b); 0 = [T,B,N]


class SruTrace(C.Structure):
    """sru_int_trace"""
    _fields_ = [("layer", C.c_int32)] + [(n, C.c_void_p) for n in SRU_TRACE_FIELDS]


_sru_ready = False


def sru_lib():
    global _sru_ready
    L = lib()
    if not _sru_ready:
        L.sru_int_prepare.restype = C.c_int
        L.sru_int_prepare.argtypes = [C.POINTER(SruLayerParams), C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
        L.sru_int_get_quant.restype = C.c_int
        L.sru_int_get_quant.argtypes = [C.c_void_p, C.c_int32, C.POINTER(SruLayerQuant)]
        L.sru_int_workspace_bytes.restype = C.c_size_t
        L.sru_int_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        L.sru_int_forward.restype = C.c_int
        L.sru_int_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(SruTrace)]
        L.sru_int_set_option.restype = C.c_int
        L.sru_int_set_option.argtypes = [C.c_void_p, C.c_char_p, C.c_int64]
        L.sru_int_profile_begin.restype = C.c_int
        L.sru_int_profile_begin.argtypes = [C.c_void_p]
        L.sru_int_profile_end.restype = C.c_int
        L.sru_int_profile_end.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_double)]
        L.sru_int_destroy.restype = None
        L.sru_int_destroy.argtypes = [C.c_void_p]
        _sru_ready = True
    return L


def marshal_sru_layers(layers):
    arr = (SruLayerParams * len(layers))()
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


class SruModel:
    """Owns one sru_int_model."""

    def __init__(self, handle, num_layers, device):
        self._h = handle
        self.num_layers = num_layers
        self.device = device

    def __del__(self):
        self.destroy()

    # sru_int_destroy
    def destroy(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.sru_int_destroy(self._h)
        self._h = None

    # sru_int_get_quant
    def get_quant(self, layer):
        q = SruLayerQuant()
        _check(sru_lib().sru_int_get_quant(self._h, layer, C.byref(q)), "sru_int_get_quant")
        N, I, G = q.N, q.I, q.G
        d = {k: getattr(q, k) for k in ("I", "N", "G", "zp_x", "zp_h", "m_c", "s_x", "s_h", "Ms", "es", "Mh", "eh")}
        for k in ("s_W", "s_v", "Mx", "ex", "Mv", "ev"):
            d[k] = list(getattr(q, k))
        d["Wq"] = _view(q.Wq, (G, N, I), np.int8)
        d["vq"] = _view(q.vq, (2, N), np.int16)
        for k in ("bq", "b_fold"):
            d[k] = _view(getattr(q, k), (G, N), np.int32)
        return d

    # sru_int_workspace_bytes
    def workspace_bytes(self, T, B):
        return sru_lib().sru_int_workspace_bytes(self._h, T, B)

    # sru_int_set_option
    def set_option(self, key, value):
        _check(sru_lib().sru_int_set_option(self._h, key.encode(), value), "sru_int_set_option")

    # sru_int_profile_begin / sru_int_profile_end
    def profile_begin(self):
        _check(sru_lib().sru_int_profile_begin(self._h), "sru_int_profile_begin")

    def profile_end(self):
        n = (C.c_int64 * 2)()
        ms = (C.c_double * 2)()
        _check(sru_lib().sru_int_profile_end(self._h, n, ms), "sru_int_profile_end")
        return {k: {"launches": int(n[i]), "total_ms": float(ms[i])} for i, k in enumerate(("input_gemm", "scan"))}

    # sru_int_forward on torch device tensors
    def forward(self, x, y=None, c_state=None, workspace=None, trace_layer=None):
        """x: int8 CUDA tensor [T,B,I0].  Returns y (int8 [T,B,N_last]); with trace_layer also a dict of
        that layer's intermediate tensors.  Asynchronous on torch's current stream."""
        import torch

        assert x.is_cuda and x.dtype == torch.int8 and x.is_contiguous()
        T, B, _ = x.shape
        ql = SruLayerQuant()
        _check(sru_lib().sru_int_get_quant(self._h, self.num_layers - 1, C.byref(ql)), "sru_int_get_quant")
        if y is None:
            y = torch.empty((T, B, ql.N), dtype=torch.int8, device=x.device)
        if workspace is None:
            workspace = torch.empty(max(self.workspace_bytes(T, B), 256), dtype=torch.uint8, device=x.device)
        tr, bufs = None, {}
        if trace_layer is not None:
            qt = SruLayerQuant()
            _check(sru_lib().sru_int_get_quant(self._h, trace_layer, C.byref(qt)), "sru_int_get_quant")
            tr = SruTrace()
            tr.layer = trace_layer
            for f, slots in SRU_TRACE_FIELDS.items():
                shape = (T, B, slots, qt.N) if slots else (T, B, qt.N)
                bufs[f] = torch.zeros(shape, dtype=torch.int8 if f == "y" else torch.int16, device=x.device)
                setattr(tr, f, bufs[f].data_ptr())
        if c_state is not None:
            assert c_state.is_cuda and c_state.dtype == torch.int16 and c_state.is_contiguous()
        stream = torch.cuda.current_stream(x.device).cuda_stream
        _check(sru_lib().sru_int_forward(self._h, x.data_ptr(), T, B, y.data_ptr(),
                                         c_state.data_ptr() if c_state is not None else None,
                                         workspace.data_ptr(), workspace.numel(), stream,
                                         C.byref(tr) if tr is not None else None), "sru_int_forward")
        return (y, bufs) if trace_layer is not None else y


# sru_int_prepare
def sru_prepare(layers, device=0):
    """layers: SruLayerSpec-like objects with their statistics filled in.  device = -1 builds a host-only model."""
    arr, keep = marshal_sru_layers(layers)
    h = C.c_void_p()
    rc = sru_lib().sru_int_prepare(arr, len(layers), device, C.byref(h))
    del keep
    _check(rc, "sru_int_prepare")
    return SruModel(h, len(layers), device)
