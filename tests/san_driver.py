"""Run by tests/test_sanitizers.py in a child process whose loader has the
AddressSanitizer runtime preloaded: drives the sanitized builds of the oracle
(LSTM_INT_ORACLE_LIB) and of the library's host arithmetic and offline phase
(argv[1]) through every variant and through the extremes of their integer
ranges.  Any out-of-bounds access, signed overflow or invalid shift aborts the
process; agreement between the two sides is asserted on the way."""
import ctypes as C
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import float_reference  # noqa: E402
import lstm_workloads as wl  # noqa: E402
import oracle  # noqa: E402
from paper_2101_05453_amd import binding  # noqa: E402  (ctypes structs only; the HIP library is not loaded)

VARIANTS = [0, wl.LAYER_NORM, wl.PEEPHOLE, wl.PROJECTION, wl.CIFG,
            wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION, wl.CIFG | wl.LAYER_NORM,
            wl.CIFG | wl.PEEPHOLE | wl.PROJECTION,
            wl.CIFG | wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION]


def checksum(model, num_layers):
    s = 0
    for l in range(num_layers):
        q = model.layer(l)
        for k in ("Wq", "Rq", "Wpq", "qb", "qbp", "bx_fold", "bh_fold", "bp_fold", "Pq", "Lq"):
            if q.get(k) is not None:
                s += int(np.asarray(q[k], dtype=np.int64).sum())
        for k in ("Mx", "ex", "Mh", "eh", "Mln", "eln"):
            s += int(sum(q[k]))
        s += q["Mm"] + q["em"] + q["Mp"] + q["ep"] + q["zp_x"] + q["zp_h"] + q["zp_m"] + q["m_c"]
    return s


def main():
    hm = C.CDLL(sys.argv[1])
    hm.hm_prepare.restype = C.c_int
    hm.hm_prepare.argtypes = [C.POINTER(binding.LayerParams), C.c_int32, C.POINTER(C.c_int64)]
    hm.hm_layernorm.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    hm.hm_layernorm2.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    hm.hm_rescale.restype = C.c_int32
    hm.hm_rescale.argtypes = [C.c_int32] * 3
    hm.hm_sigmoid_table.argtypes = [C.c_int, C.c_void_p]
    hm.hm_tanh_table.argtypes = [C.c_int, C.c_void_p]
    hm.hm_cell_update32.argtypes = [C.c_int32] * 5
    hm.hm_hidden.argtypes = [C.c_int32] * 5
    oracle.lib()

    # 1. every variant: both offline phases, then the oracle's forward with every trace and saturating inputs
    for flags in VARIANTS:
        H = 24 if flags & wl.PROJECTION else 56
        layers, x = wl.make_custom([36, H], 56, H, flags, 4, 8, seed=flags + 3, weight_param=0.2)
        float_reference.collect_statistics(layers, x)
        arr, keep = binding.marshal_layers(layers)
        cs = C.c_int64()
        assert hm.hm_prepare(arr, len(layers), C.byref(cs)) == 0
        om = oracle.prepare(layers)
        assert cs.value == checksum(om, len(layers)), (flags, cs.value)
        q0 = om.layer(0)
        xq = oracle.quantize_input(x * 3, q0["s_x"], q0["zp_x"])
        for l in range(2):
            oracle.forward(om, xq, trace_layer=l)
        oracle.forward(om, xq, unfolded=True)
        oracle.forward(om, xq, reverse=True)
        oracle.float_forward(layers, x)
    print("variants ok", flush=True)

    # 2. layer norm at its row limit with extreme rows (all +32767; alternating +-32767; one spike), both sides
    n = 4096
    rows = [np.full(n, 32767, np.int16), np.where(np.arange(n) % 2 == 0, 32767, -32767).astype(np.int16),
            np.where(np.arange(n) == 7, -32768, 0).astype(np.int16), np.full(n, -32768, np.int16)]
    qL = np.where(np.arange(n) % 3 == 0, 32767, -32767).astype(np.int16)
    qb = np.where(np.arange(n) % 2 == 0, 2**31 - 1, -(2**31 - 1)).astype(np.int32)
    for M, e in ((2**30, 1), (2**31 - 1, -5), (1518500250, -20)):
        for q in rows:
            want = oracle.int_layernorm(q, qL, qb, M, e)
            for fn in (hm.hm_layernorm, hm.hm_layernorm2) if 31 - e >= 32 else (hm.hm_layernorm,):
                out = np.zeros(n, np.int16)
                fn(q.ctypes.data, n, qL.ctypes.data, qb.ctypes.data, M, 31 - e, out.ctypes.data)
                assert (out == want).all(), (M, e)
    print("layer norm extremes ok", flush=True)

    # 3. accumulation depth 2^15 with weights and inputs at their bounds (Sec. 3.1.1), and a layer-norm model at N = 4096
    layers, x = wl.make_custom([32768], 16, 16, 0, 2, 2, seed=9, weight_param=0.01)
    float_reference.collect_statistics(layers, x)
    for g in range(4):  # every weight at +-max so that the quantized ones are all +-127
        layers[0].W[g] = np.where(layers[0].W[g] >= 0, 0.01, -0.01).astype(np.float32)
    om = oracle.prepare(layers)
    arr, keep = binding.marshal_layers(layers)
    cs = C.c_int64()
    assert hm.hm_prepare(arr, 1, C.byref(cs)) == 0 and cs.value == checksum(om, 1)
    xq = np.where(np.asarray(layers[0].W[1][0])[None, None, :] >= 0, -128, 127).astype(np.int8).repeat(2, 0).repeat(2, 1)
    oracle.forward(om, np.ascontiguousarray(xq), trace_layer=0)
    layers, x = wl.make_custom([16], 4096, 4096, wl.LAYER_NORM, 2, 2, seed=8, weight_param=0.02)
    float_reference.collect_statistics(layers, x)
    om = oracle.prepare(layers)
    q0 = om.layer(0)
    oracle.forward(om, oracle.quantize_input(x * 50, q0["s_x"], q0["zp_x"]), trace_layer=0)
    print("depth and width limits ok", flush=True)

    # 4. scalar helpers at the corners of their domains
    for a in (-2**31, -1, 0, 1, 2**31 - 1):
        for M in (2**30, 2**31 - 1):
            for e in (-31, -1, 0, 30):
                assert hm.hm_rescale(a, M, 31 - e) == oracle.rescale(a, M, e)
    tab = np.zeros(32769, np.uint16)
    for m in range(9):
        hm.hm_sigmoid_table(m, tab.ctypes.data)
        hm.hm_tanh_table(m, tab.ctypes.data)
        for v in (-32768, -1, 0, 1, 32767):
            oracle.int_sigmoid(v, m), oracle.int_tanh(v, m)
    for m_c in range(9):
        for i, z, f, c in ((32767, 32767, 32767, 32767), (32767, -32768, 32767, -32768), (0, 0, 0, 0)):
            hm.hm_cell_update32(i, z, f, c, m_c)
    # 5. the GRU of the same oracle: ragged shapes, saturating inputs and gate sums, depth 2^15 at the weight bounds
    from oracle import gru  # noqa: E402

    layers, x = wl.make_gru([19, 37], 37, 3, 9, seed=6, weight_param=0.3, input_dist="uniform", input_param=3.0)
    layers[0].x_min, layers[0].x_max = -1.0, 2.0
    layers[0].bx[1] = layers[0].bx[1] * 80
    gm = gru.GruModel(layers)
    q0 = gm.get_quant(0)
    xq = np.clip(np.floor(x.astype(np.float64) / q0["s_x"] + 0.5) + q0["zp_x"], -128, 127).astype(np.int8)
    hs = np.full(2 * 3 * 37, -32768, np.int16)
    for l in range(2):
        gm.forward(xq, h_state=hs, trace_layer=l)
    gm.forward(xq, unfolded=True)
    gru.float_forward(layers, x)
    layers, x = wl.make_gru([32768], 8, 1, 2, seed=2, weight_param=0.01)
    for g in range(3):
        layers[0].W[g] = np.where(layers[0].W[g] >= 0, 0.01, -0.01).astype(np.float32)
    gm = gru.GruModel(layers)
    xq = np.where(np.asarray(layers[0].W[0][0])[None, None, :] >= 0, -128, 127).astype(np.int8).repeat(2, 0)
    gm.forward(np.ascontiguousarray(xq), trace_layer=0)
    print("gru ok", flush=True)
    # 6. the SRU of the same oracle: both forms of the highway term, ragged shapes, saturating values, a state at its bounds
    from oracle import sru  # noqa: E402

    layers, x = wl.make_sru([19, 37, 37], 37, 3, 9, seed=6, weight_param=0.3, input_dist="uniform", input_param=3.0)
    sru.calibrate(layers, x)
    layers[0].x_min, layers[0].x_max = -1.0, 2.0
    for s in layers:
        s.b[0] = s.b[0] * 40
        s.c_absmax *= 0.25
        s.h_max *= 0.2
    sm = sru.SruModel(layers)
    q0 = sm.get_quant(0)
    xq = np.clip(np.floor(x.astype(np.float64) / q0["s_x"] + 0.5) + q0["zp_x"], -128, 127).astype(np.int8)
    cs = np.full(3 * 3 * 37, -32768, np.int16)
    for l in range(3):
        sm.forward(xq, c_state=cs, trace_layer=l)
    sm.forward(xq, unfolded=True)
    layers, x = wl.make_sru([32768], 8, 1, 2, seed=2, weight_param=0.01)
    for g in range(4):
        layers[0].W[g] = np.where(layers[0].W[g] >= 0, 0.01, -0.01).astype(np.float32)
    sru.calibrate(layers, x)
    sm = sru.SruModel(layers)
    xq = np.where(np.asarray(layers[0].W[0][0])[None, None, :] >= 0, -128, 127).astype(np.int8).repeat(2, 0)
    sm.forward(np.ascontiguousarray(xq), trace_layer=0)
    print("sru ok", flush=True)
    print("SAN DRIVER OK", flush=True)


if __name__ == "__main__":
    main()
