"""The library's offline phase of the integer GRU (gru_int_prepare, host-only model) against the
oracle's: every quantized tensor, zero point, scale and (M, e) pair identical; argument checks as
include/gru_int.h states them; the library exports every symbol that header declares.  No GPU."""
import os
import re

import numpy as np
import pytest

import lstm_workloads as wl
from paper_2101_05453_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SHAPES = [([24], 40, 0.2), ([32, 64], 64, 0.1), ([17, 37, 37], 37, 0.3), ([640, 1024], 1024, 0.03)]


def test_library_exports_every_declared_gru_symbol():
    text = open(os.path.join(ROOT, "include", "gru_int.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(gru_int_[a-z_]+)\s*\(", text)))
    assert names == ["gru_int_destroy", "gru_int_device_status", "gru_int_forward", "gru_int_get_quant", "gru_int_prepare",
                     "gru_int_profile_begin", "gru_int_profile_end", "gru_int_set_option", "gru_int_workspace_bytes"]
    lib = binding.gru_lib()
    for n in names:
        assert hasattr(lib, n), n


def test_struct_layout_matches_header_field_order():
    text = open(os.path.join(ROOT, "include", "gru_int.h")).read()
    for cname, cls in (("gru_int_layer_params", binding.GruLayerParams), ("gru_int_layer_quant", binding.GruLayerQuant),
                       ("gru_int_trace", binding.GruTrace)):
        body = re.search(r"typedef struct \{([^}]*)\} %s;" % cname, text, re.S).group(1)
        body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
        fields = []
        for decl in body.split(";"):
            decl = decl.strip()
            if decl:
                for name in decl.split(","):
                    fields.append(re.sub(r"\[.*", "", name.strip().split()[-1].lstrip("*")))
        assert fields == [f[0] for f in cls._fields_], cname


@pytest.mark.parametrize("shape", SHAPES)
def test_prepare_matches_oracle(orc, shape):
    from oracle import gru

    inputs, N, wp = shape
    layers, x = wl.make_gru(inputs, N, 2, 3, seed=13, weight_param=wp, input_dist="uniform", input_param=2.5)
    layers[0].x_min *= 0.7  # zero point away from the middle
    a = binding.gru_prepare(layers, device=-1)
    b = gru.GruModel(layers)
    for l in range(len(layers)):
        qa, qb = a.get_quant(l), b.get_quant(l)
        assert set(qa) == set(qb)
        for k in qa:
            if isinstance(qa[k], np.ndarray):
                assert qa[k].dtype == qb[k].dtype and (qa[k] == qb[k]).all(), (l, k)
            else:
                assert qa[k] == qb[k], (l, k)


def test_argument_checks():
    layers, _ = wl.make_gru([16, 24], 24, 1, 1)
    ok = binding.gru_prepare(layers, device=-1)
    assert ok.workspace_bytes(4, 3) > 0
    import ctypes as C

    buf = (C.c_int8 * 1024)()
    with pytest.raises(binding.LstmIntError) as e:  # a host-only model cannot run
        binding._check(binding.gru_lib().gru_int_forward(ok._h, buf, 1, 1, buf, None, buf, 1 << 20, None, None), "fw")
    assert e.value.code == binding.E_DEVICE
    bad, _ = wl.make_gru([16, 30], 24, 1, 1)
    with pytest.raises(binding.LstmIntError) as e:
        binding.gru_prepare(bad, device=-1)
    assert e.value.code == binding.E_INVALID_ARG
    bad, _ = wl.make_gru([16], 24, 1, 1)
    bad[0].R[2] = bad[0].R[2].copy()
    bad[0].R[2][3, 3] = np.inf
    with pytest.raises(binding.LstmIntError) as e:
        binding.gru_prepare(bad, device=-1)
    assert e.value.code == binding.E_BAD_RANGE
    bad, _ = wl.make_gru([16], 24, 1, 1)
    bad[0].x_min, bad[0].x_max = 1.0, -1.0
    with pytest.raises(binding.LstmIntError) as e:
        binding.gru_prepare(bad, device=-1)
    assert e.value.code == binding.E_BAD_RANGE
    bad, _ = wl.make_gru([16], 24, 1, 1)
    bad[0].bh[0] = np.full(24, 3e9, np.float32)  # bias + 128 sum|w| leaves int32
    with pytest.raises(binding.LstmIntError) as e:
        binding.gru_prepare(bad, device=-1)
    assert e.value.code == binding.E_UNSUPPORTED
