"""Pins of the oracle's prepare and forward: Table 2 ranges, the zero-point
identity of Sec. 6, the plain matmul definition, stage-by-stage exact
rational checks on traces, agreement with the float LSTM of Sec. 2 within the
quantization error, split sequences, and the limits prepare enforces.
"""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import lstm_workloads as wl

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))

VARIANTS = [0, wl.LAYER_NORM, wl.PEEPHOLE, wl.PROJECTION, wl.CIFG,
            wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION,
            wl.CIFG | wl.LAYER_NORM, wl.CIFG | wl.PEEPHOLE | wl.PROJECTION,
            wl.CIFG | wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION]


def rhu_fr(fr):
    return math.floor(fr + Fraction(1, 2))


def sat(v, bits):
    return max(-(1 << (bits - 1)), min((1 << (bits - 1)) - 1, v))


def py_rescale(a, M, e):
    return sat(rhu_fr(Fraction(a * M, 1 << (31 - e))), 32)


def calibrated(orc, layers, x):
    yf, stats = orc.float_forward(layers, x)
    orc.apply_stats(layers, stats)
    return yf, stats


def small(flags, L=1, I=24, N=40, H=16, B=3, T=6, seed=5, **kw):
    return wl.make_custom([I] + [H if flags & wl.PROJECTION else N] * (L - 1), N, H, flags, B, T,
                          seed=seed, **kw)


# ---------------------------------------------------------------- prepare
@pytest.mark.parametrize("flags", VARIANTS)
def test_prepare_follows_table2(orc, flags):
    layers, x = small(flags, weight_param=0.2)
    calibrated(orc, layers, x)
    q = orc.prepare(layers).layer(0)
    s = layers[0]
    first = 1 if flags & wl.CIFG else 0
    for g in range(first, 4):
        for key, src, lim in (("Wq", s.W[g], "weight_range"), ("Rq", s.R[g], "weight_range")):
            t = q[key][g]
            assert t.min() >= GOLD[lim]["lo"] and t.max() <= GOLD[lim]["hi"]
            assert np.abs(t).max() == 127  # the largest magnitude maps to the end of the range
            sc = np.abs(src).astype(np.float64).max() / 127.0
            assert q["s_W" if key == "Wq" else "s_R"][g] == sc
            assert np.abs(t * sc - src).max() <= sc / 2 * (1 + 1e-9)
    if first:
        assert not q["Wq"][0].any() and not q["Rq"][0].any()
    # asymmetric activations: real 0 is a code, the range is covered
    for nm, lo, hi in (("x", s.x_min, s.x_max), ("h", s.h_min, s.h_max)):
        sc, zp = q["s_" + nm], q["zp_" + nm]
        assert GOLD["activation_range"]["lo"] <= zp <= GOLD["activation_range"]["hi"]
        lo, hi = min(np.float32(lo), 0.0), max(np.float32(hi), 0.0)
        assert sc == (float(hi) - float(lo)) / 255.0
        assert abs(sc * (-128 - zp) - lo) <= sc / 2 + 1e-12 and abs(sc * (127 - zp) - hi) <= sc / 2 + 1e-12
    if not flags & wl.PROJECTION:
        assert (q["s_m"], q["zp_m"]) == (q["s_h"], q["zp_h"])
    # cell: power-of-two scale covering the measured range (Sec. 3.2.2)
    assert q["s_c"] == 2.0 ** (q["m_c"] - 15)
    assert 2.0 ** q["m_c"] >= np.float32(s.c_absmax) and (q["m_c"] == 0 or 2.0 ** (q["m_c"] - 1) < np.float32(s.c_absmax))
    for g in range(first, 4):
        if flags & wl.LAYER_NORM:
            assert q["s_g"][g] == float(np.float32(s.g_absmax[g])) / 32767.0
            assert np.abs(q["Lq"][g]).max() == 32767
            sb = 2.0**-10 * q["s_L"][g]
        else:
            assert q["s_g"][g] == 2.0**-12
            sb = q["s_R"][g] * q["s_h"]
        assert np.abs(q["qb"][g] * sb - s.b[g]).max() <= sb / 2 * (1 + 1e-9)
        for key, seff in (("x", q["s_W"][g] * q["s_x"] / q["s_g"][g]), ("h", q["s_R"][g] * q["s_h"] / q["s_g"][g])):
            M, e = q["M" + key][g], q["e" + key][g]
            assert abs(M * 2.0 ** (e - 31) / seff - 1) < 2.0**-30
    if flags & wl.PEEPHOLE:
        for j in range(first, 3):
            assert np.abs(q["Pq"][j]).max() == 32767
    M, e = q["Mm"], q["em"]
    assert abs(M * 2.0 ** (e - 31) / (2.0**-30 / q["s_m"]) - 1) < 2.0**-30


def test_prepare_folds_zero_points_exactly(orc):
    """Sec. 6: sum W (q - zp) + b = sum W q + b' as integers."""
    layers, x = small(wl.PROJECTION, weight_param=0.2)
    calibrated(orc, layers, x)
    q = orc.prepare(layers).layer(0)
    for g in range(4):
        assert (q["bx_fold"][g] == -q["zp_x"] * q["Wq"][g].astype(np.int64).sum(1)).all()
        assert (q["bh_fold"][g] == q["qb"][g] - q["zp_h"] * q["Rq"][g].astype(np.int64).sum(1)).all()
    assert (q["bp_fold"] == q["qbp"] - q["zp_m"] * q["Wpq"].astype(np.int64).sum(1)).all()


def test_cell_format_example_from_the_paper(orc):
    """Sec. 3.2.2: a cell in [-3.2, 10] is extended to [-16, 16): Q4.11."""
    ex = GOLD["cell_format_example"]
    layers, x = small(0)
    calibrated(orc, layers, x)
    layers[0].c_absmax = max(abs(v) for v in ex["range"])
    q = orc.prepare(layers).layer(0)
    assert q["m_c"] == ex["m"] and q["s_c"] == 2.0 ** -ex["n"] and ex["m"] + ex["n"] == 15
    for c, m in ((0.3, 0), (1.0, 0), (1.0001, 1), (8.0, 3), (8.5, 4), (255.0, 8)):
        layers[0].c_absmax = c
        assert orc.prepare(layers).layer(0)["m_c"] == m
    layers[0].c_absmax = 257.0
    with pytest.raises(orc.OracleError) as ei:
        orc.prepare(layers)
    assert ei.value.code == orc.UNSUPPORTED


def test_prepare_saturates_at_the_table2_bounds(orc):
    layers, x = small(wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION)
    calibrated(orc, layers, x)
    s = layers[0]
    s.b[1] = s.b[1].copy()
    s.b[1][0], s.b[1][1] = 1e9, -1e9  # far beyond int32 at scale 2^-10 s_L
    q = orc.prepare(layers).layer(0)
    assert q["qb"][1][0] == GOLD["bias_range"]["hi"] and q["qb"][1][1] == GOLD["bias_range"]["lo"]
    for key in ("Pq", "Lq"):
        assert q[key].min() >= GOLD["int16_weight_range"]["lo"] and q[key].max() <= GOLD["int16_weight_range"]["hi"]


def test_prepare_rejects_bad_arguments(orc):
    def fresh(flags=0):
        layers, x = small(flags)
        calibrated(orc, layers, x)
        return layers

    def code(layers):
        with pytest.raises(orc.OracleError) as ei:
            orc.prepare(layers)
        return ei.value.code

    l = fresh(wl.CIFG)
    l[0].W[0] = np.zeros((40, 24), np.float32)  # a dagger row of Table 2 under CIFG
    assert code(l) == orc.INVALID_ARG
    l = fresh()
    l[0].R[2] = None
    assert code(l) == orc.INVALID_ARG
    l = fresh()
    l[0].P[0] = np.zeros(40, np.float32)  # peephole weights without the flag
    assert code(l) == orc.INVALID_ARG
    l = fresh()
    l[0].output_size = 16  # no projection: H must equal N
    assert code(l) == orc.INVALID_ARG
    l = fresh()
    l[0].h_min, l[0].h_max = 1.0, -1.0
    assert code(l) == orc.BAD_RANGE
    l = fresh()
    l[0].W[1] = l[0].W[1].copy()
    l[0].W[1][0, 0] = np.nan
    assert code(l) == orc.BAD_RANGE
    # a bias so large that bias + worst-case accumulation leaves int32
    l = fresh()
    l[0].b[3] = l[0].b[3].copy()
    l[0].b[3][5] = 1e6
    assert code(l) == orc.UNSUPPORTED


def test_accumulation_depth_limit(orc):
    """Sec. 3.1.1: int8 x int8 -> int32 is safe for 2^15 steps; the extreme
    product (-127)(-128) summed 2^15 times, plus the folded zero-point term of
    the same size, still fits."""
    assert GOLD["safe_depth_int32"]["log2_steps"] == 15
    K = 2**15
    assert K * 127 * 128 + 128 * K * 127 <= 2**31 - 1
    # the paper's depths count a product of two 8-bit values as 16 bits:
    # a signed w-bit accumulator holds 2^(w-1) = depth * 2^16
    assert GOLD["safe_depth_int32"]["log2_steps"] == 32 - 1 - 16
    assert GOLD["safe_depth_24bit"]["log2_steps"] == 24 - 1 - 16
    layers, x = wl.make_custom([K + 16], 4, 4, 0, 1, 1)
    calibrated(orc, layers, x)
    with pytest.raises(orc.OracleError) as ei:
        orc.prepare(layers)
    assert ei.value.code == orc.UNSUPPORTED


def test_adversarial_matmul_at_full_depth(orc):
    """All weights -127 against all inputs -128 at K = 2048 (and the safe
    depth 2^15): the traced W x term equals the int64 definition."""
    for K in (2048, 2**15):
        layers, x = wl.make_custom([K], 2, 2, 0, 1, 1)
        for g in range(4):
            layers[0].W[g][:] = -1.0
        calibrated(orc, layers, x)
        layers[0].x_min, layers[0].x_max = -1.0, 0.0  # zp_x = 127: q = -128 is real -1
        layers[0].h_min, layers[0].h_max, layers[0].c_absmax = -1.0, 1.0, 1.0
        m = orc.prepare(layers)
        q = m.layer(0)
        assert (q["Wq"] == -127).all() and q["zp_x"] == 127
        xq = np.full((1, 1, K), -128, np.int8)
        _, tr = orc.forward(m, xq, trace_layer=0)
        acc = K * 127 * 128 + int(q["bx_fold"][0][0])
        assert acc == K * (-127) * (-128 - 127)
        assert tr["tx"][0, 0, 0, 0] == sat(py_rescale(acc, q["Mx"][0], q["ex"][0]), 16)


# ---------------------------------------------------------------- forward, stage by stage
@pytest.mark.parametrize("flags", VARIANTS)
def test_forward_stages_against_exact_arithmetic(orc, flags):
    """Each traced stage is recomputed from the stage before it with numpy
    int64 matmuls and exact rationals."""
    layers, x = small(flags, L=2, weight_param=0.15, seed=flags + 1)
    calibrated(orc, layers, x)
    m = orc.prepare(layers)
    q0 = m.layer(0)
    xq = orc.quantize_input(x, q0["s_x"], q0["zp_x"])
    T, B, _ = xq.shape
    _, tr0 = orc.forward(m, xq, trace_layer=0)
    y, tr1 = orc.forward(m, xq, trace_layer=1)
    assert (y == tr1["h"]).all()
    cifg, ph = bool(flags & wl.CIFG), bool(flags & wl.PEEPHOLE)
    ln, proj = bool(flags & wl.LAYER_NORM), bool(flags & wl.PROJECTION)
    for l, (tr, xin) in enumerate(((tr0, xq), (tr1, tr0["h"]))):
        q = m.layer(l)
        N, H = q["N"], q["H"]
        for t in range(T):
            for b in range(B):
                hp = tr["h"][t - 1, b] if t else np.full(H, q["zp_h"], np.int8)
                cp = tr["c"][t - 1, b].astype(np.int64) if t else np.zeros(N, np.int64)
                cn = tr["c"][t, b].astype(np.int64)
                for g in range(1 if cifg else 0, 4):
                    accx = q["Wq"][g].astype(np.int64) @ xin[t, b].astype(np.int64) + q["bx_fold"][g]
                    acch = q["Rq"][g].astype(np.int64) @ hp.astype(np.int64) + q["bh_fold"][g]
                    for n in range(0, N, 7):
                        tx = sat(py_rescale(int(accx[n]), q["Mx"][g], q["ex"][g]), 16)
                        th = sat(py_rescale(int(acch[n]), q["Mh"][g], q["eh"][g]), 16)
                        assert (tx, th) == (tr["tx"][t, b, g, n], tr["th"][t, b, g, n])
                        tc = 0
                        if ph and g != 2:
                            j = 2 if g == 3 else g
                            cc = int(cn[n]) if g == 3 else int(cp[n])  # o reads c^t (eq. 5)
                            tc = sat(py_rescale(int(q["Pq"][j][n]) * cc, q["Mc"][j], q["ec"][j]), 16)
                        want = max(-32767 if ln else -32768, min(32767, tx + th + tc))
                        assert want == tr["g"][t, b, g, n]
                    gin = tr["g"][t, b, g]
                    if ln:
                        gin = orc.int_layernorm(gin, q["Lq"][g], q["qb"][g], q["Mln"][g], q["eln"][g])
                        assert (gin == tr["ln"][t, b, g]).all()
                    f = orc.int_tanh if g == 2 else orc.int_sigmoid
                    assert [f(int(v), 3) for v in gin] == tr["act"][t, b, g].tolist()
                a = tr["act"][t, b].astype(np.int64)
                for n in range(N):
                    i = min(32768 - int(a[1, n]), 32767) if cifg else int(a[0, n])
                    assert i == a[0, n]
                    cw = sat(rhu_fr(Fraction(i * int(a[2, n]), 1 << (15 + q["m_c"])))
                             + rhu_fr(Fraction(int(a[1, n]) * int(cp[n]), 1 << 15)), 16)
                    assert cw == cn[n]
                    mw = sat(py_rescale(int(a[3, n]) * orc.int_tanh(int(cn[n]), q["m_c"]), q["Mm"], q["em"])
                             + q["zp_m"], 8)
                    assert mw == tr["m"][t, b, n]
                if proj:
                    acc = q["Wpq"].astype(np.int64) @ tr["m"][t, b].astype(np.int64) + q["bp_fold"]
                    hw = [sat(py_rescale(int(v), q["Mp"], q["ep"]) + q["zp_h"], 8) for v in acc]
                    assert hw == tr["h"][t, b].tolist()
                else:
                    assert (tr["h"][t, b] == tr["m"][t, b]).all()
        if cifg:  # Sec. 3.2.9: the coupled input gate lies in [1, 32767]
            lim = GOLD["cifg_input_gate_range"]
            assert tr["act"][:, :, 0].min() >= lim["lo"] and tr["act"][:, :, 0].max() <= lim["hi"]


@pytest.mark.parametrize("flags", VARIANTS)
def test_folded_equals_unfolded(orc, flags):
    layers, x = small(flags, L=2, seed=9)
    calibrated(orc, layers, x)
    m = orc.prepare(layers)
    q0 = m.layer(0)
    xq = orc.quantize_input(x, q0["s_x"], q0["zp_x"])
    y1, t1 = orc.forward(m, xq, trace_layer=1)
    y2, t2 = orc.forward(m, xq, trace_layer=1, unfolded=True)
    assert (y1 == y2).all()
    for k in t1:
        assert (t1[k] == t2[k]).all(), k


def test_gate_sum_saturates_at_both_bounds(orc):
    """Q3.12 gate sum clamps to [-32768, 32767] without layer norm
    (Sec. 3.2.4) and to [-32767, 32767] with it (Sec. 3.2.5)."""
    for flags, key in ((0, "gate_q3_12_range"), (wl.LAYER_NORM, "gate_ln_range")):
        layers, x = small(flags, weight_param=0.3, I=64)
        calibrated(orc, layers, x)
        if flags:
            layers[0].g_absmax = [0.05] * 4  # far too small a measured range: saturates
        else:
            for g in range(4):
                layers[0].W[g] *= 40.0
        m = orc.prepare(layers)
        q0 = m.layer(0)
        xq = orc.quantize_input(x * 3, q0["s_x"], q0["zp_x"])
        assert xq.min() == -128 and xq.max() == 127
        _, tr = orc.forward(m, xq, trace_layer=0)
        assert tr["g"].min() == GOLD[key]["lo"] and tr["g"].max() == GOLD[key]["hi"]
        assert tr["tx"].min() == -32768 and tr["tx"].max() == 32767


def test_hidden_and_cell_saturate(orc):
    layers, x = small(wl.PROJECTION, weight_param=0.4)
    calibrated(orc, layers, x)
    layers[0].m_min, layers[0].m_max = -0.01, 0.01
    layers[0].h_min, layers[0].h_max = -0.01, 0.02
    layers[0].c_absmax = 0.5
    m = orc.prepare(layers)
    q0 = m.layer(0)
    xq = orc.quantize_input(x, q0["s_x"], q0["zp_x"])
    _, tr = orc.forward(m, xq, trace_layer=0)
    assert tr["m"].min() == -128 and tr["m"].max() == 127
    assert tr["h"].min() == -128 and tr["h"].max() == 127
    # f = 32767, i = 0 cannot move the cell by more than one step per update
    for c in (-32768, -5, 0, 77, 32767):
        assert abs(rhu_fr(Fraction(32767 * c, 1 << 15)) - c) <= 1


# ---------------------------------------------------------------- against the float LSTM
def _agreement(orc, layers, x):
    yf, _ = calibrated(orc, layers, x)
    m = orc.prepare(layers)
    q0, ql = m.layer(0), m.layer(m.num_layers - 1)
    xq = orc.quantize_input(x, q0["s_x"], q0["zp_x"])
    y = orc.forward(m, xq)
    err = np.abs((y.astype(np.float64) - ql["zp_h"]) * ql["s_h"] - yf) / ql["s_h"]
    return err


@pytest.mark.parametrize("name,B,T,L,mean_tol,max_tol", [
    ("C1", 1, 20, 1, 0.6, 3.0),
    ("C2", 4, 100, 1, 1.0, 12.0),
    ("C3", 2, 24, 1, 1.2, 10.0),
    ("C4", 2, 12, 1, 1.2, 10.0),
    ("C5", 2, 12, 1, 1.5, 14.0),
])
def test_integer_lstm_tracks_float_lstm(orc, name, B, T, L, mean_tol, max_tol):
    """Error against the double LSTM of Sec. 2 in units of the output step
    s_h.  The paper gives no numeric bound beyond Sec. 3.2.1; these bands were
    measured with the oracle and then frozen (about twice the measured value).
    A wrong shift, sign, gate order or transposed operand gives tens of
    steps."""
    layers, x = wl.make_workload(name, batch=B, steps=T, num_layers=L)
    err = _agreement(orc, layers, x)
    assert err.mean() <= mean_tol and err.max() <= max_tol, (err.mean(), err.max())


@pytest.mark.parametrize("flags", VARIANTS)
def test_every_variant_tracks_float(orc, flags):
    layers, x = wl.make_custom([48], 96, 40, flags, 3, 30, seed=flags, weight_param=0.1)
    err = _agreement(orc, layers, x)
    assert err.mean() <= 1.5 and err.max() <= 12.0, (flags, err.mean(), err.max())


@pytest.mark.parametrize("flags", [wl.PEEPHOLE, wl.PEEPHOLE | wl.LAYER_NORM, wl.PEEPHOLE | wl.CIFG])
def test_strong_peephole_tracks_float(orc, flags):
    """Peephole weights twenty times the benchmark's, distinct per gate, so
    that a wrong peephole slot, scale, or cell-state time index (i and f read
    c^{t-1}, o reads c^t, z reads none: eqs. 1-5) costs far more than the
    band."""
    layers, x = wl.make_custom([48], 96, 96, flags, 3, 30, seed=40 + flags, weight_param=0.1)
    for j, k in enumerate((20.0, -14.0, 8.0)):
        if layers[0].P[j] is not None:
            layers[0].P[j] = (np.abs(layers[0].P[j]) * k).astype(np.float32)
    err = _agreement(orc, layers, x)
    assert err.mean() <= 1.5 and err.max() <= 12.0, (flags, err.mean(), err.max())


def test_error_does_not_grow_over_long_sequences(orc):
    """Sec. 5 reports robustness on 16.5-minute utterances; errors may
    accumulate in time (Sec. 1).  Mean error over the last quarter of a long
    sequence stays at the level of the first quarter."""
    layers, x = wl.make_custom([32], 64, 64, wl.LAYER_NORM, 2, 2000, seed=3, weight_param=0.1)
    yf, _ = calibrated(orc, layers, x)
    m = orc.prepare(layers)
    q = m.layer(0)
    y = orc.forward(m, orc.quantize_input(x, q["s_x"], q["zp_x"]))
    err = np.abs((y.astype(np.float64) - q["zp_h"]) * q["s_h"] - yf) / q["s_h"]
    first, last = err[:500].mean(), err[-500:].mean()
    assert last <= 1.5 * first + 0.2 and err.mean() <= 1.5, (first, last)


def test_stacked_layers_feed_scales_forward(orc):
    layers, x = wl.make_workload("C4", batch=2, steps=6, num_layers=3)
    calibrated(orc, layers, x)
    m = orc.prepare(layers)
    for l in (1, 2):
        assert (m.layer(l)["s_x"], m.layer(l)["zp_x"]) == (m.layer(l - 1)["s_h"], m.layer(l - 1)["zp_h"])


# ---------------------------------------------------------------- state carrying, shapes
@pytest.mark.parametrize("flags", [0, wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION, wl.CIFG | wl.LAYER_NORM])
def test_split_sequence_equals_one_call(orc, flags):
    layers, x = small(flags, L=2, T=10, seed=21)
    calibrated(orc, layers, x)
    m = orc.prepare(layers)
    q0 = m.layer(0)
    xq = orc.quantize_input(x, q0["s_x"], q0["zp_x"])
    B = xq.shape[1]
    dims = m.dims()
    y = orc.forward(m, xq)
    hs = np.concatenate([np.full(B * d[2], m.layer(l)["zp_h"], np.int8) for l, d in enumerate(dims)])
    cs = np.zeros(sum(B * d[1] for d in dims), np.int16)
    ya = orc.forward(m, xq[:4], h_state=hs, c_state=cs)
    yb = orc.forward(m, xq[4:], h_state=hs, c_state=cs)
    assert (np.concatenate([ya, yb]) == y).all()
    # the final state is the last h of each layer
    assert (hs[-B * dims[-1][2]:].reshape(B, -1) == y[-1]).all()


def test_rows_are_independent(orc):
    """No cross-row term anywhere (eqs. 1-7; layer norm is per row): a subset
    of batch rows gives the same rows."""
    layers, x = small(wl.LAYER_NORM | wl.PROJECTION, L=2, B=5)
    calibrated(orc, layers, x)
    m = orc.prepare(layers)
    q0 = m.layer(0)
    xq = orc.quantize_input(x, q0["s_x"], q0["zp_x"])
    y = orc.forward(m, xq, threads=3)
    sub = orc.forward(m, np.ascontiguousarray(xq[:, [4, 1]]), threads=1)
    assert (sub == y[:, [4, 1]]).all()


def test_empty_inputs(orc):
    layers, x = small(0)
    calibrated(orc, layers, x)
    m = orc.prepare(layers)
    assert orc.forward(m, np.zeros((0, 3, 24), np.int8)).shape == (0, 3, 40)
    assert orc.forward(m, np.zeros((4, 0, 24), np.int8)).shape == (4, 0, 40)


def test_reverse_direction_runs_backward_in_time(orc):
    """In the backward direction the output at time t depends on x[t..T-1] only:
    changing x[0] leaves y[1:] alone, changing x[T-1] reaches y[0]; and with one
    step the two directions coincide."""
    import lstm_workloads as wl
    import float_reference

    layers, x = wl.make_custom([12], 16, 16, wl.LAYER_NORM, 3, 6, seed=4)
    float_reference.collect_statistics(layers, x)
    model = orc.prepare(layers)
    q = model.layer(0)
    xq = orc.quantize_input(x, q["s_x"], q["zp_x"])
    y = orc.forward(model, xq, reverse=True)
    x2 = xq.copy()
    x2[0] = np.where(x2[0] > 0, x2[0] - 37, x2[0] + 37)
    y2 = orc.forward(model, x2, reverse=True)
    assert np.array_equal(y2[1:], y[1:]) and not np.array_equal(y2[0], y[0])
    x3 = xq.copy()
    x3[-1] = np.where(x3[-1] > 0, x3[-1] - 37, x3[-1] + 37)
    y3 = orc.forward(model, x3, reverse=True)
    assert not np.array_equal(y3[0], y[0])
    # the forward direction has the opposite dependence
    yf, yf2 = orc.forward(model, xq), orc.forward(model, x2)
    assert not np.array_equal(yf2[-1], yf[-1])
    assert np.array_equal(orc.forward(model, xq[:1], reverse=True), orc.forward(model, xq[:1]))
