"""The C-ABI library loads, exports every symbol include/lstm_int.h declares,
and its host-side logic (argument checks, host-only prepare) behaves as the
header states.  No GPU work here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import lstm_workloads as wl
import float_reference
from paper_2101_05453_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "lstm_int.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lstm_int_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.lib()
    names = declared_symbols()
    assert {"lstm_int_prepare", "lstm_int_forward", "lstm_int_get_quant", "lstm_int_workspace_bytes",
            "lstm_int_destroy", "lstm_int_strerror", "lstm_int_set_option", "lstm_int_profile_begin",
            "lstm_int_profile_end"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_names_match_header():
    for n in declared_symbols():
        short = n[len("lstm_int_"):]
        assert hasattr(binding, short) or hasattr(binding.Model, short) or short in ("destroy", "forward"), n


def test_struct_layouts_match_header_field_order():
    text = open(os.path.join(ROOT, "include", "lstm_int.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} lstm_int_layer_params;", text, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in body.split(";"):
        decl = decl.strip()
        if decl:
            for name in decl.split(","):
                fields.append(re.sub(r"\[.*", "", name.strip().split()[-1].lstrip("*")))
    assert fields == [f[0] for f in binding.LayerParams._fields_]


def test_strerror_and_error_codes():
    assert binding.strerror(0) == "ok"
    for code in range(-6, 0):
        assert binding.strerror(code) not in ("ok", "unknown error")
    assert binding.strerror(-99) == "unknown error"


def _calibrated(flags=0, **kw):
    layers, x = wl.make_custom([24], 40, 16, flags, 3, 6, seed=1, **kw)
    float_reference.collect_statistics(layers, x)
    return layers, x


def test_host_only_model_and_argument_checks():
    layers, x = _calibrated(wl.LAYER_NORM | wl.PROJECTION)
    m = binding.prepare(layers, device=-1)
    q = m.get_quant(0)
    assert (q["I"], q["N"], q["H"], q["G"]) == (24, 40, 16, 4)
    assert m.workspace_bytes(6, 3) > 0 and m.workspace_bytes(0, 3) == 256
    with pytest.raises(binding.LstmIntError) as ei:
        m.get_quant(1)
    assert ei.value.code == binding.E_INVALID_ARG
    # a host-only model cannot run
    buf = np.zeros(4096, np.int8)
    with pytest.raises(binding.LstmIntError) as ei:
        m.forward_ptr(buf.ctypes.data, 1, 1, buf.ctypes.data, None, None, buf.ctypes.data, 4096, None)
    assert ei.value.code == binding.E_DEVICE
    with pytest.raises(binding.LstmIntError) as ei:
        m.set_option("no-such-key", 1)
    assert ei.value.code == binding.E_INVALID_ARG
    m.set_option("path", 1)
    with pytest.raises(binding.LstmIntError):
        m.set_option("path", 99)
    lib = binding.lib()
    assert lib.lstm_int_prepare(None, 1, -1, None) == binding.E_INVALID_ARG
    h = C.c_void_p()
    assert lib.lstm_int_prepare(None, 1, -1, C.byref(h)) == binding.E_INVALID_ARG and not h.value
    lib.lstm_int_destroy(None)  # a no-op


def test_prepare_error_codes():
    def code(layers):
        with pytest.raises(binding.LstmIntError) as ei:
            binding.prepare(layers, device=-1)
        return ei.value.code

    l, _ = _calibrated(wl.CIFG)
    l[0].W[0] = np.zeros((40, 24), np.float32)
    assert code(l) == binding.E_INVALID_ARG
    l, _ = _calibrated()
    l[0].output_size = 16
    assert code(l) == binding.E_INVALID_ARG
    l, _ = _calibrated()
    l[0].h_min, l[0].h_max = 1.0, -1.0
    assert code(l) == binding.E_BAD_RANGE
    l, _ = _calibrated()
    l[0].R[3] = l[0].R[3].copy()
    l[0].R[3][1, 1] = np.inf
    assert code(l) == binding.E_BAD_RANGE
    l, _ = _calibrated()
    l[0].c_absmax = 1000.0
    assert code(l) == binding.E_UNSUPPORTED
    l, _ = _calibrated()
    l[0].b[3] = l[0].b[3].copy()
    l[0].b[3][5] = 1e6  # bias + worst-case accumulation leaves int32
    assert code(l) == binding.E_UNSUPPORTED
    layers, x = wl.make_custom([24], 5000, 5000, wl.LAYER_NORM, 1, 1)
    for s in layers:
        s.h_min, s.h_max, s.x_min, s.x_max, s.c_absmax, s.g_absmax = -1, 1, -1, 1, 1.0, [1.0] * 4
    assert code(layers) == binding.E_UNSUPPORTED  # N > 4096 with layer norm
    two, _ = wl.make_custom([24, 40], 40, 40, 0, 1, 1)
    two[1].input_size = 41
    assert code(two) == binding.E_INVALID_ARG


def test_calibrate_rejects_bad_arguments_before_touching_a_device():
    lib = binding.lib()
    layers, x = wl.make_custom([8], 16, 16, 0, 2, 2, seed=1)
    arr, keep = binding.marshal_layers(layers)
    st = (binding.LayerStats * 1)()
    dummy = C.c_void_p(256)  # never dereferenced: every call below fails its argument checks first
    assert lib.lstm_int_calibrate(arr, 0, 0, dummy, 2, 2, None, st, None) == -1
    assert lib.lstm_int_calibrate(arr, 1, 0, None, 2, 2, None, st, None) == -1
    assert lib.lstm_int_calibrate(arr, 1, 0, dummy, 0, 2, None, st, None) == -1
    assert lib.lstm_int_calibrate(arr, 1, -1, dummy, 2, 2, None, st, None) == -1
    assert lib.lstm_int_calibrate(arr, 1, 0, dummy, 2, 2, None, None, None) == -1
    arr[0].output_size = 12  # without PROJECTION the output width is the cell count
    assert lib.lstm_int_calibrate(arr, 1, 0, dummy, 2, 2, None, st, None) == -1
    arr[0].output_size = 16
    arr[0].num_cells = arr[0].output_size = 1 << 20  # T * B * 4 * N beyond the 32-bit index range
    assert lib.lstm_int_calibrate(arr, 1, 0, dummy, 1 << 10, 2, None, st, None) == -2
    del keep


def test_lds_probe_rejects_arguments_outside_its_array():
    """The probe's addresses stay inside its LDS array only for the documented ranges; everything else is refused on
    the host, before any device call."""
    lib = binding.lib()
    for args in ((0, 3, 16, 0, 0), (0, -1, 16, 0, 0), (0, 0, 132, 0, 0), (0, 0, 0, 0, 0), (0, 0, 18, 0, 0), (0, 0, 16, 3, 0),
                 (-1, 0, 16, 0, 0)):
        assert lib.lstm_int_lds_probe(*args) == binding.E_INVALID_ARG, args
