"""Pins of the oracle's integer GRU (oracle/gru_int_oracle.c).

Sec. 7 of arXiv 2101.05453 names the GRU as a user of the paper's building blocks and gives no
recipe: what the oracle computes is this build's reading (stated in gru_int_oracle.h), "parity
unpinned" by the paper.  What can be pinned is: the float cell against a library GRU
(torch.nn.GRU has the same form), every integer stage against exact rational arithmetic written
out here, the quantization against Table 2's rules, the zero-point identity of Sec. 6, closed
forms of degenerate cells, agreement with the float cell within the quantization error with no
growth over long sequences, and state carrying.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

import lstm_workloads as wl


@pytest.fixture(scope="module")
def gru(orc):
    from oracle import gru as g

    g.lib()
    return g


def rhu_fr(fr):
    return math.floor(fr + Fraction(1, 2))


def sat(v, bits):
    return max(-(1 << (bits - 1)), min((1 << (bits - 1)) - 1, v))


def py_rescale(a, M, e):
    return sat(rhu_fr(Fraction(a * M, 1 << (31 - e))), 32)


def quantize_x(x, q):
    return np.clip(np.floor(x.astype(np.float64) / q["s_x"] + 0.5) + q["zp_x"], -128, 127).astype(np.int8)


def torch_gru(layers, x):
    """The library's GRU in float64 with the same parameters (its gate order is r, z, n with
    z the update gate; n = tanh(W_in x + b_in + r * (W_hn h + b_hn)); h' = (1 - z) n + z h)."""
    N = layers[0].num_cells
    inp = torch.from_numpy(x).to(torch.float64)
    for s in layers:
        m = torch.nn.GRU(s.input_size, N, num_layers=1).to(torch.float64)
        with torch.no_grad():
            m.weight_ih_l0.copy_(torch.from_numpy(np.concatenate(s.W)).to(torch.float64))
            m.weight_hh_l0.copy_(torch.from_numpy(np.concatenate(s.R)).to(torch.float64))
            m.bias_ih_l0.copy_(torch.from_numpy(np.concatenate(s.bx)).to(torch.float64))
            m.bias_hh_l0.copy_(torch.from_numpy(np.concatenate(s.bh)).to(torch.float64))
            inp, _ = m(inp)
    return inp.numpy()


def test_float_gru_matches_library_gru(gru):
    layers, x = wl.make_gru([20, 36, 36], 36, 4, 15, seed=3, weight_param=0.3)
    y = gru.float_forward(layers, x, threads=2)
    ref = torch_gru(layers, x)
    assert np.abs(y - ref).max() < 1e-12


def test_prepare_follows_the_quantization_rules(gru):
    layers, x = wl.make_gru([24, 40], 40, 3, 6, seed=5, weight_param=0.2)
    m = gru.GruModel(layers)
    for l, s in enumerate(layers):
        q = m.get_quant(l)
        for g in range(3):
            for key, src, sk in (("Wq", s.W[g], "s_W"), ("Rq", s.R[g], "s_R")):
                t = q[key][g]
                assert t.min() >= -127 and t.max() <= 127 and np.abs(t).max() == 127  # Sec. 3.2.4: +-127
                sc = Fraction(float(np.abs(src).astype(np.float64).max())) / 127
                assert q[sk][g] == pytest.approx(float(sc), rel=1e-15)
                want = np.array([sat(rhu_fr(Fraction(float(v)) / Fraction(q[sk][g])), 8) for v in src.ravel()[:500]])
                assert (t.ravel()[:500] == np.clip(want, -127, 127)).all()
        if l == 0:
            # asymmetric int8 with the range widened to 0 and a nudged zero point (Sec. 3.2.4)
            lo, hi = min(s.x_min, 0.0), max(s.x_max, 0.0)
            assert q["s_x"] == pytest.approx((hi - lo) / 255.0, rel=1e-15)
            assert q["zp_x"] == sat(rhu_fr(Fraction(-128) - Fraction(float(np.float32(lo))) / Fraction(q["s_x"])), 8)
        else:
            assert q["s_x"] == 2.0 ** -7 and q["zp_x"] == 0  # the int8 form of the state below
        for g in range(3):
            # biases at the scale of their accumulators; effective scales to Q3.12
            sbx, sbh = Fraction(q["s_W"][g]) * Fraction(q["s_x"]), Fraction(q["s_R"][g]) / 128
            for n in range(0, 40, 7):
                assert q["bxq"][g][n] == rhu_fr(Fraction(float(s.bx[g][n])) / sbx)
                assert q["bhq"][g][n] == rhu_fr(Fraction(float(s.bh[g][n])) / sbh)
            for (M, e), sc in (((q["Mx"][g], q["ex"][g]), sbx * 4096), ((q["Mh"][g], q["eh"][g]), sbh * 4096)):
                assert 2 ** 30 <= M < 2 ** 31
                assert abs(Fraction(M) * Fraction(2) ** (e - 31) / sc - 1) <= Fraction(1, 2 ** 31)
            # zero point folded into the input bias (Sec. 6)
            fold = q["bxq"][g].astype(np.int64) - q["zp_x"] * q["Wq"][g].astype(np.int64).sum(axis=1)
            assert (q["bx_fold"][g] == fold).all()


def test_every_stage_against_exact_rationals(gru, orc):
    layers, x = wl.make_gru([24, 40], 40, 2, 5, seed=7, weight_param=0.25, input_param=1.5)
    m = gru.GruModel(layers)
    xq = quantize_x(x, m.get_quant(0))
    y0, tr0 = m.forward(xq, trace_layer=0)
    for l, inp in ((0, xq), (1, tr0["h8"])):
        q = m.get_quant(l)
        y, tr = m.forward(xq, trace_layer=l)
        T, B, _ = inp.shape
        N = q["N"]
        h16 = np.zeros((B, N), dtype=np.int64)
        h8 = np.zeros((B, N), dtype=np.int64)
        for t in range(T):
            for b in range(B):
                xv = inp[t, b].astype(np.int64)
                new16 = np.zeros(N, dtype=np.int64)
                for n in range(0, N, 3):  # a third of the cells, every gate
                    tx, th = [], []
                    for g in range(3):
                        ax = int((q["Wq"][g][n].astype(np.int64) * (xv - q["zp_x"])).sum()) + int(q["bxq"][g][n])
                        ah = int((q["Rq"][g][n].astype(np.int64) * h8[b]).sum()) + int(q["bhq"][g][n])
                        tx.append(sat(py_rescale(ax, q["Mx"][g], q["ex"][g]), 16))
                        th.append(sat(py_rescale(ah, q["Mh"][g], q["eh"][g]), 16))
                        assert tr["tx"][t, b, g, n] == tx[g] and tr["th"][t, b, g, n] == th[g]
                    r = orc.int_sigmoid(sat(tx[0] + th[0], 16), 3)
                    u = orc.int_sigmoid(sat(tx[1] + th[1], 16), 3)
                    rn = rhu_fr(Fraction(r * th[2], 1 << 15))
                    c = orc.int_tanh(sat(tx[2] + rn, 16), 3)
                    ubar = min(32768 - u, 32767)
                    hn = sat(rhu_fr(Fraction(ubar * c, 1 << 15)) + rhu_fr(Fraction(u * int(h16[b, n]), 1 << 15)), 16)
                    assert (tr["act"][t, b, :, n] == [r, u, c]).all()
                    assert tr["h16"][t, b, n] == hn
                    assert tr["h8"][t, b, n] == sat(rhu_fr(Fraction(hn, 256)), 8)
                new16[:] = tr["h16"][t, b]
                h16[b] = new16
                h8[b] = tr["h8"][t, b]
        if l == 1:
            assert (y == tr["h8"]).all()


def test_folded_equals_unfolded(gru):
    layers, x = wl.make_gru([33, 48], 48, 3, 9, seed=11, weight_param=0.2, input_dist="uniform", input_param=3.0)
    layers[0].x_min = 0.5 * layers[0].x_min  # a range that clips some inputs, and a zero point away from 0
    m = gru.GruModel(layers)
    assert m.get_quant(0)["zp_x"] != 0
    xq = quantize_x(x, m.get_quant(0))
    ya, _ = m.forward(xq)
    yb, _ = m.forward(xq, unfolded=True)
    assert (ya == yb).all()


def test_degenerate_cell_halves_its_state(gru):
    """All parameters zero: r = u = sigma(0) = 1/2, n = tanh(0) = 0, so h' = h / 2, rounded half up."""
    N = 8
    z = wl.GruLayerSpec(4, N, [np.zeros((N, 4), np.float32)] * 3, [np.zeros((N, N), np.float32)] * 3,
                        [np.zeros(N, np.float32)] * 3, [np.zeros(N, np.float32)] * 3, -1.0, 1.0)
    m = gru.GruModel([z])
    h = np.array([[32767, -32768, 1, -1, 3, -3, 1000, 0]], dtype=np.int16)
    want = h.astype(np.int64).copy()
    xq = np.zeros((6, 1, 4), dtype=np.int8)
    y, tr = m.forward(xq, h_state=h, trace_layer=0)
    for t in range(6):
        want = (want * 16384 + 16384) >> 15  # rsh_r(16384 h, 15); the other product is 16384 * 0
        assert (tr["h16"][t, 0] == want[0]).all()
        assert (tr["act"][t, 0, 0] == 16384).all() and (tr["act"][t, 0, 1] == 16384).all() and (tr["act"][t, 0, 2] == 0).all()
    assert (h == want).all()  # the state buffer carries the last state


def test_saturated_update_gate_keeps_the_state(gru):
    """bx_u far beyond the Q3.12 range: the gate sum saturates at 32767, u = sigma(~8) and the coupled
    1 - u = 32768 - u (Sec. 3.2.9); the state moves by the closed form below."""
    N = 4
    zero_w, zero_r, zero_b = np.zeros((N, 2), np.float32), np.zeros((N, N), np.float32), np.zeros(N, np.float32)
    big = np.full(N, 1000.0, np.float32)
    s = wl.GruLayerSpec(2, N, [zero_w] * 3, [zero_r] * 3, [zero_b, big, zero_b], [zero_b] * 3, -1.0, 1.0)
    m = gru.GruModel([s])
    h = np.array([[20000, -20000, 5, 0]], dtype=np.int16)
    h_in = h.astype(np.int64).copy()
    _, tr = m.forward(np.zeros((1, 1, 2), dtype=np.int8), h_state=h, trace_layer=0)
    assert (tr["tx"][0, 0, 1] == 32767).all()  # saturated, Sec. 3.2.4
    u = int(tr["act"][0, 0, 1, 0])
    assert u == round(32768 / (1 + math.exp(-32767 / 4096)))
    want = (u * h_in + 16384) >> 15  # n = 0
    assert (h == want).all() and np.abs(want - h_in).max() <= 12


@pytest.mark.parametrize("T", [20, 400])
def test_agrees_with_the_float_gru(gru, T):
    layers, x = wl.make_gru([32, 64], 64, 4, T, seed=2, weight_param=0.1)
    m = gru.GruModel(layers)
    xq = quantize_x(x, m.get_quant(0))
    y, _ = m.forward(xq, threads=4)
    yf = gru.float_forward(layers, x, threads=4)
    err = np.abs(y.astype(np.float64) * 2.0 ** -7 - yf) * 128  # in LSB of the int8 output
    # measured: mean 0.5-0.7 LSB, max 3-4 LSB; no growth along the sequence (the state is 16 bits wide)
    assert err.mean() < 1.0 and err.max() < 6.0
    if T >= 400:
        assert err[-50:].mean() < 1.5 * err[:50].mean() + 0.2


def test_split_sequence_carries_state(gru):
    layers, x = wl.make_gru([16, 24], 24, 3, 14, seed=9, weight_param=0.3)
    m = gru.GruModel(layers)
    xq = quantize_x(x, m.get_quant(0))
    hs = np.zeros(2 * 3 * 24, dtype=np.int16)
    whole, _ = m.forward(xq, h_state=hs)
    hs2 = np.zeros_like(hs)
    a, _ = m.forward(xq[:5], h_state=hs2)
    b, _ = m.forward(xq[5:], h_state=hs2)
    assert (np.concatenate([a, b]) == whole).all() and (hs == hs2).all()
    none, _ = m.forward(xq)
    assert (none == whole).all()  # no state buffer = zeros


def test_rows_are_independent_and_limits_hold(gru):
    from oracle import OracleError

    layers, x = wl.make_gru([16], 24, 5, 7, seed=4, weight_param=0.3)
    m = gru.GruModel(layers)
    xq = quantize_x(x, m.get_quant(0))
    y, _ = m.forward(xq, threads=3)
    for b in range(5):
        yb, _ = m.forward(xq[:, b:b + 1])
        assert (yb[:, 0] == y[:, b]).all()
    bad = wl.make_gru([16], 24, 1, 1)[0]
    bad[0].W[1] = bad[0].W[1].copy()
    bad[0].W[1][0, 0] = np.nan
    with pytest.raises(OracleError):
        gru.GruModel(bad)
    bad = wl.make_gru([16, 30], 24, 1, 1)[0]  # layer 1 does not read layer 0's width
    with pytest.raises(OracleError):
        gru.GruModel(bad)
