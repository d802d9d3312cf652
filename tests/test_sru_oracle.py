"""Pins of the oracle's integer SRU (oracle/sru_int_oracle.c).

Sec. 7 of arXiv 2101.05453 names the SRU as a user of the paper's building blocks and gives no
recipe: what the oracle computes is this build's reading (stated in sru_int_oracle.h), "parity
unpinned" by the paper.  What can be pinned is: the float cell against library routines in the
cases that reduce to them (constant gates make the state a first-order recursive filter:
scipy.signal.lfilter), the roles of the two recurrent weight vectors through what they must do to
the state, every integer stage against exact rational arithmetic written out here, the
quantization against Table 2's rules, the zero-point identity of Sec. 6, closed forms of
degenerate cells, agreement with the float cell within the quantization error with no growth over
long sequences, and state carrying.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
from scipy.signal import lfilter

import lstm_workloads as wl


@pytest.fixture(scope="module")
def sru(orc):
    from oracle import sru as s

    s.lib()
    return s


def rhu_fr(fr):
    return math.floor(fr + Fraction(1, 2))


def sat(v, bits):
    return max(-(1 << (bits - 1)), min((1 << (bits - 1)) - 1, v))


def py_rescale(a, M, e):
    return sat(rhu_fr(Fraction(a * M, 1 << (31 - e))), 32)


def quantize_x(x, q):
    return np.clip(np.floor(x.astype(np.float64) / q["s_x"] + 0.5) + q["zp_x"], -128, 127).astype(np.int8)


def logit(p):
    return np.log(p / (1.0 - p)).astype(np.float32)


def test_constant_gates_make_the_state_a_recursive_filter(sru):
    """W_f = W_r = 0, v = 0: f = sigma(b_f) = p and r = sigma(b_r) = q per cell, so
    c_t = p c_{t-1} + (1 - p) (W_c x_t) is lfilter([1 - p], [1, -p]) along time and
    h_t = q c_t + (1 - q) s_t -- with the new state, and s = W_s x or x itself."""
    rng = np.random.default_rng(0)
    for with_s in (True, False):
        I, N, B, T = (11, 7, 3, 25) if with_s else (7, 7, 3, 25)
        layers, x = wl.make_sru([I], N, B, T, seed=1, weight_param=0.4, highway_matrix=with_s)
        s = layers[0]
        p, q = rng.uniform(0.1, 0.9, N), rng.uniform(0.1, 0.9, N)
        s.W[1], s.W[2] = np.zeros_like(s.W[1]), np.zeros_like(s.W[2])
        s.v = [np.zeros(N, np.float32), np.zeros(N, np.float32)]
        s.b = [logit(p), logit(q)]
        p, q = 1 / (1 + np.exp(-s.b[0].astype(np.float64))), 1 / (1 + np.exp(-s.b[1].astype(np.float64)))
        y, stats = sru.float_forward(layers, x)
        xd = x.astype(np.float64)
        xc = xd @ s.W[0].astype(np.float64).T
        hw = xd @ s.W[3].astype(np.float64).T if with_s else xd
        c = np.stack([lfilter([1 - p[n]], [1, -p[n]], xc[:, :, n], axis=0) for n in range(N)], axis=-1)
        ref = q * c + (1 - q) * hw
        assert np.abs(y - ref).max() < 1e-12
        assert stats[0]["c_absmax"] == pytest.approx(max(np.abs(c).max(), np.abs(xc).max(), np.abs(hw).max()), rel=1e-12)
        assert stats[0]["h_min"] == pytest.approx(min(ref.min(), 0.0), rel=1e-12)
        assert stats[0]["h_max"] == pytest.approx(max(ref.max(), 0.0), rel=1e-12)


def test_recurrent_vectors_gate_on_the_old_state_of_their_own_cell(sru):
    """v_f large on a cell whose candidate is positive: from step 2 on f = sigma(v_f c_1 + ...) ~ 1 and the
    state stays where step 1 left it -- c_1 = (1 - sigma(b_f)) xc_1 exactly, because the gate of step 1 saw
    the old state 0, not the new one.  v_r large instead: the state filters on, and h ~ c from step 2 on.
    Other cells are untouched: the vectors act per cell."""
    I, N, B, T = 5, 6, 2, 12
    layers, x = wl.make_sru([I], N, B, T, seed=2, weight_param=0.3)
    s = layers[0]
    x = np.abs(x) + 0.5
    s.W[0] = np.abs(s.W[0])  # candidates positive
    s.W[1], s.W[2] = np.zeros_like(s.W[1]), np.zeros_like(s.W[2])
    s.b = [np.zeros(N, np.float32), np.zeros(N, np.float32)]
    base_v = [np.zeros(N, np.float32), np.zeros(N, np.float32)]
    s.v = [v.copy() for v in base_v]
    y0, _ = sru.float_forward(layers, x)
    xc = x.astype(np.float64) @ s.W[0].astype(np.float64).T
    hw = x.astype(np.float64) @ s.W[3].astype(np.float64).T
    # v_f on cell 2
    s.v = [v.copy() for v in base_v]
    s.v[0][2] = 400.0
    y1, _ = sru.float_forward(layers, x)
    c1 = 0.5 * xc[0, :, 2]  # sigma(0) = 1/2 at step 1: the gate read c_0 = 0
    assert np.abs(y1[1:, :, 2] - (0.5 * c1 + 0.5 * hw[1:, :, 2])).max() < 1e-9  # frozen state, r = 1/2
    others = [n for n in range(N) if n != 2]
    assert (y1[:, :, others] == y0[:, :, others]).all()
    # v_r on cell 4
    s.v = [v.copy() for v in base_v]
    s.v[1][4] = 400.0
    y2, _ = sru.float_forward(layers, x)
    c = lfilter([0.5], [1, -0.5], xc[:, :, 4], axis=0)
    assert np.abs(y2[0, :, 4] - (0.5 * c[0] + 0.5 * hw[0, :, 4])).max() < 1e-12  # step 1: r = sigma(0)
    assert np.abs(y2[1:, :, 4] - c[1:]).max() < 1e-9  # r ~ 1: h = the new state
    others = [n for n in range(N) if n != 4]
    assert (y2[:, :, others] == y0[:, :, others]).all()


def test_prepare_follows_the_quantization_rules(sru):
    layers, x = wl.make_sru([24, 40], 40, 3, 6, seed=5, weight_param=0.2)
    sru.calibrate(layers, x)
    m = sru.SruModel(layers)
    prev = None
    for l, s in enumerate(layers):
        q = m.get_quant(l)
        G = 4 if s.W[3] is not None else 3
        assert q["G"] == G and (G == 4) == (l == 0)
        # state format: the smallest power of two that holds the measured magnitude (Sec. 3.2.2)
        assert 2.0 ** q["m_c"] >= np.float32(s.c_absmax) and (q["m_c"] == 0 or 2.0 ** (q["m_c"] - 1) < np.float32(s.c_absmax))
        s_c = Fraction(2) ** (q["m_c"] - 15)
        for g in range(G):
            t = q["Wq"][g]
            assert t.min() >= -127 and t.max() <= 127 and np.abs(t).max() == 127  # Sec. 3.2.4: +-127
            sc = Fraction(float(np.abs(s.W[g]).astype(np.float64).max())) / 127
            assert q["s_W"][g] == pytest.approx(float(sc), rel=1e-15)
            want = np.array([sat(rhu_fr(Fraction(float(v)) / Fraction(q["s_W"][g])), 8) for v in s.W[g].ravel()[:500]])
            assert (t.ravel()[:500] == np.clip(want, -127, 127)).all()
        for j in range(2):  # recurrent vectors: 16 bits, +-32767 (Sec. 3.2.3)
            t = q["vq"][j]
            assert np.abs(t).max() == 32767
            assert q["s_v"][j] == pytest.approx(float(np.abs(s.v[j]).astype(np.float64).max()) / 32767, rel=1e-15)
            assert (t == [sat(rhu_fr(Fraction(float(v)) / Fraction(q["s_v"][j])), 16) for v in s.v[j]]).all()
            M, e = q["Mv"][j], q["ev"][j]
            assert 2 ** 30 <= M < 2 ** 31
            assert abs(Fraction(M) * Fraction(2) ** (e - 31) / (Fraction(q["s_v"][j]) * s_c * 4096) - 1) <= Fraction(1, 2 ** 31)
        if l == 0:
            lo, hi = min(s.x_min, 0.0), max(s.x_max, 0.0)
            assert q["s_x"] == pytest.approx((hi - lo) / 255.0, rel=1e-15)
            assert q["zp_x"] == sat(rhu_fr(Fraction(-128) - Fraction(float(np.float32(lo))) / Fraction(q["s_x"])), 8)
        else:
            assert q["s_x"] == prev["s_h"] and q["zp_x"] == prev["zp_h"]  # reads the output of the layer below
        lo, hi = min(np.float32(s.h_min), 0.0), max(np.float32(s.h_max), 0.0)
        assert q["s_h"] == pytest.approx((float(hi) - float(lo)) / 255.0, rel=1e-15)
        assert q["zp_h"] == sat(rhu_fr(Fraction(-128) - Fraction(float(lo)) / Fraction(q["s_h"])), 8)
        for g in range(G):
            sb = Fraction(q["s_W"][g]) * Fraction(q["s_x"])
            gate = g in (1, 2)
            for n in range(0, 40, 7):
                assert q["bq"][g][n] == (rhu_fr(Fraction(float(s.b[g - 1][n])) / sb) if gate else 0)
            target = Fraction(1, 4096) if gate else s_c  # gates to Q3.12, candidate and highway to the state's format
            M, e = q["Mx"][g], q["ex"][g]
            assert 2 ** 30 <= M < 2 ** 31
            assert abs(Fraction(M) * Fraction(2) ** (e - 31) / (sb / target) - 1) <= Fraction(1, 2 ** 31)
            fold = q["bq"][g].astype(np.int64) - q["zp_x"] * q["Wq"][g].astype(np.int64).sum(axis=1)
            assert (q["b_fold"][g] == fold).all()  # Sec. 6
        if G == 3:
            assert abs(Fraction(q["Ms"]) * Fraction(2) ** (q["es"] - 31) / (Fraction(q["s_x"]) / s_c) - 1) <= Fraction(1, 2 ** 31)
        assert abs(Fraction(q["Mh"]) * Fraction(2) ** (q["eh"] - 31) / (s_c / Fraction(q["s_h"])) - 1) <= Fraction(1, 2 ** 31)
        prev = q


def test_every_stage_against_exact_rationals(sru, orc):
    layers, x = wl.make_sru([24, 40], 40, 2, 5, seed=7, weight_param=0.25, input_param=1.5)
    sru.calibrate(layers, x)
    m = sru.SruModel(layers)
    xq = quantize_x(x, m.get_quant(0))
    _, tr0 = m.forward(xq, trace_layer=0)
    for l, inp in ((0, xq), (1, tr0["y"])):  # layer 0 has W_s, layer 1 takes its input as the highway term
        q = m.get_quant(l)
        y, tr = m.forward(xq, trace_layer=l)
        T, B, _ = inp.shape
        N, G = q["N"], q["G"]
        c = np.zeros((B, N), dtype=np.int64)
        for t in range(T):
            for b in range(B):
                xv = inp[t, b].astype(np.int64)
                for n in range(0, N, 3):  # a third of the cells, every slot
                    tx = []
                    for g in range(G):
                        a = int((q["Wq"][g][n].astype(np.int64) * (xv - q["zp_x"])).sum()) + int(q["bq"][g][n])
                        tx.append(sat(py_rescale(a, q["Mx"][g], q["ex"][g]), 16))
                    if G == 3:
                        tx.append(sat(py_rescale(int(xv[n]) - q["zp_x"], q["Ms"], q["es"]), 16))
                    assert (tr["tx"][t, b, :, n] == tx).all()
                    tv = [sat(py_rescale(int(q["vq"][j][n]) * int(c[b, n]), q["Mv"][j], q["ev"][j]), 16) for j in range(2)]
                    assert (tr["tv"][t, b, :, n] == tv).all()
                    f = orc.int_sigmoid(sat(tx[1] + tv[0], 16), 3)
                    r = orc.int_sigmoid(sat(tx[2] + tv[1], 16), 3)
                    assert (tr["act"][t, b, :, n] == [f, r]).all()
                    fbar, rbar = min(32768 - f, 32767), min(32768 - r, 32767)
                    cn = sat(rhu_fr(Fraction(f * int(c[b, n]), 1 << 15)) + rhu_fr(Fraction(fbar * tx[0], 1 << 15)), 16)
                    hn = sat(rhu_fr(Fraction(r * cn, 1 << 15)) + rhu_fr(Fraction(rbar * tx[3], 1 << 15)), 16)
                    assert tr["c"][t, b, n] == cn and tr["h16"][t, b, n] == hn
                    assert tr["y"][t, b, n] == sat(py_rescale(hn, q["Mh"], q["eh"]) + q["zp_h"], 8)
                c[b] = tr["c"][t, b]
        if l == 1:
            assert (y == tr["y"]).all()


def test_folded_equals_unfolded(sru):
    layers, x = wl.make_sru([33, 48], 48, 3, 9, seed=11, weight_param=0.2, input_dist="uniform", input_param=3.0)
    sru.calibrate(layers, x)
    layers[0].x_min = 0.5 * layers[0].x_min  # a range that clips some inputs, and a zero point away from 0
    m = sru.SruModel(layers)
    assert m.get_quant(0)["zp_x"] != 0 and m.get_quant(1)["zp_x"] != 0
    xq = quantize_x(x, m.get_quant(0))
    ya, _ = m.forward(xq)
    yb, _ = m.forward(xq, unfolded=True)
    assert (ya == yb).all()


def zero_layer(I, N, with_s, b_f=0.0):
    W = [np.zeros((N, I), np.float32) for _ in range(4 if with_s else 3)] + ([] if with_s else [None])
    return wl.SruLayerSpec(I, N, W, [np.zeros(N, np.float32)] * 2,
                           [np.full(N, b_f, np.float32), np.zeros(N, np.float32)], -1.0, 1.0, 1.0, -1.0, 1.0)


def test_degenerate_cell_halves_its_state(sru):
    """All parameters zero: f = r = sigma(0) = 1/2 and the candidate and the highway term are 0, so
    c' = c / 2 and h = c' / 2, each rounded half up; the output is h at 2^-15 over the scale 2 / 255."""
    N = 8
    m = sru.SruModel([zero_layer(4, N, True)])
    q = m.get_quant(0)
    assert q["m_c"] == 0 and q["zp_h"] == 0
    c = np.array([[32767, -32768, 1, -1, 3, -3, 1000, 0]], dtype=np.int16)
    want = c.astype(np.int64).copy()
    y, tr = m.forward(np.zeros((6, 1, 4), dtype=np.int8), c_state=c, trace_layer=0)
    for t in range(6):
        want = (want * 16384 + 16384) >> 15
        h = (want * 16384 + 16384) >> 15
        assert (tr["act"][t, 0] == 16384).all() and (tr["tx"][t, 0] == 0).all()
        assert (tr["c"][t, 0] == want[0]).all() and (tr["h16"][t, 0] == h[0]).all()
        assert (y[t, 0] == [sat(rhu_fr(Fraction(int(v), 1 << 15) / (Fraction(2) / 255)), 8) for v in h[0]]).all()
    assert (c == want).all()  # the state buffer carries the last state


def test_saturated_forget_gate_keeps_the_state(sru):
    """b_f far beyond the Q3.12 range: the gate term saturates at 32767, f = sigma(~8) and the coupled
    1 - f = 32768 - f (Sec. 3.2.9); with a zero candidate the state moves by the closed form below."""
    N = 4
    m = sru.SruModel([zero_layer(2, N, True, b_f=1000.0)])
    c = np.array([[20000, -20000, 5, 0]], dtype=np.int16)
    c_in = c.astype(np.int64).copy()
    _, tr = m.forward(np.zeros((1, 1, 2), dtype=np.int8), c_state=c, trace_layer=0)
    assert (tr["tx"][0, 0, 1] == 32767).all()  # saturated, Sec. 3.2.4
    f = int(tr["act"][0, 0, 0, 0])
    assert f == round(32768 / (1 + math.exp(-32767 / 4096)))
    want = (f * c_in + 16384) >> 15
    assert (c == want).all() and np.abs(want - c_in).max() <= 12


def test_identity_highway_passes_the_input(sru):
    """No W_s, r's bias very negative: r = sigma(-8) ~ 0, so h ~ x: the output, on the input's own grid
    (h range = x range), reproduces the input codes to within a code."""
    N = 16
    s = zero_layer(N, N, False)
    s.b = [np.zeros(N, np.float32), np.full(N, -1000.0, np.float32)]
    s.x_min, s.x_max, s.h_min, s.h_max, s.c_absmax = -2.0, 6.0, -2.0, 6.0, 6.0
    m = sru.SruModel([s])
    q = m.get_quant(0)
    assert q["G"] == 3 and q["m_c"] == 3 and q["zp_h"] == q["zp_x"]
    xq = np.arange(-128, 128, dtype=np.int8).reshape(16, 1, 16)
    y, tr = m.forward(xq, trace_layer=0)
    s16 = tr["tx"][:, :, 3]  # the input at 2^-12
    exact = (xq.astype(np.float64) - q["zp_x"]) * q["s_x"] * 4096
    assert np.abs(s16 - exact).max() <= 0.5 + 1e-6
    assert np.abs(y.astype(np.int64) - xq).max() <= 1


@pytest.mark.parametrize("T", [20, 400])
def test_agrees_with_the_float_sru(sru, T):
    layers, x = wl.make_sru([32, 64, 64], 64, 4, T, seed=2, weight_param=0.1)
    yf = sru.calibrate(layers, x, threads=4)
    m = sru.SruModel(layers)
    xq = quantize_x(x, m.get_quant(0))
    y, _ = m.forward(xq, threads=4)
    q = m.get_quant(2)
    err = np.abs((y.astype(np.float64) - q["zp_h"]) * q["s_h"] - yf) / q["s_h"]  # in LSB of the int8 output
    # three layers of 8-bit activations; no growth along the sequence (the state is 16 bits wide)
    assert err.mean() < 1.5 and err.max() < 8.0
    if T >= 400:
        assert err[-50:].mean() < 1.5 * err[:50].mean() + 0.2


def test_split_sequence_carries_state(sru):
    layers, x = wl.make_sru([16, 24], 24, 3, 14, seed=9, weight_param=0.3)
    sru.calibrate(layers, x)
    m = sru.SruModel(layers)
    xq = quantize_x(x, m.get_quant(0))
    cs = np.zeros(2 * 3 * 24, dtype=np.int16)
    whole, _ = m.forward(xq, c_state=cs)
    cs2 = np.zeros_like(cs)
    a, _ = m.forward(xq[:5], c_state=cs2)
    b, _ = m.forward(xq[5:], c_state=cs2)
    assert (np.concatenate([a, b]) == whole).all() and (cs == cs2).all()
    none, _ = m.forward(xq)
    assert (none == whole).all()  # no state buffer = zeros


def test_rows_are_independent_and_limits_hold(sru):
    from oracle import OracleError

    layers, x = wl.make_sru([16], 24, 5, 7, seed=4, weight_param=0.3)
    sru.calibrate(layers, x)
    m = sru.SruModel(layers)
    xq = quantize_x(x, m.get_quant(0))
    y, _ = m.forward(xq, threads=3)
    for b in range(5):
        yb, _ = m.forward(xq[:, b:b + 1])
        assert (yb[:, 0] == y[:, b]).all()
    bad = wl.make_sru([16], 24, 1, 1)[0]
    bad[0].W[1] = bad[0].W[1].copy()
    bad[0].W[1][0, 0] = np.nan
    with pytest.raises(OracleError):
        sru.SruModel(bad)
    bad = wl.make_sru([16, 30], 24, 1, 1)[0]  # layer 1 does not read layer 0's width
    with pytest.raises(OracleError):
        sru.SruModel(bad)
    bad = wl.make_sru([16], 24, 1, 1, highway_matrix=False)[0]  # the input cannot be the highway term: 16 != 24
    with pytest.raises(OracleError):
        sru.SruModel(bad)
    bad = wl.make_sru([16], 24, 1, 1)[0]
    bad[0].c_absmax = 300.0  # beyond Q8.7
    with pytest.raises(OracleError):
        sru.SruModel(bad)
