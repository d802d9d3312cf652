"""Pins of the oracle's fixed-point primitives against what the paper and the
mathematics fix: exact rational arithmetic, libm in double, defining
inequalities, and the numbers the paper prints (tests/golden/paper_values.json).
"""
import json
import math
import os
import random
from fractions import Fraction

import numpy as np
import pytest

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


def exact_round_half_up(fr):
    """floor(fr + 1/2) for a Fraction."""
    return math.floor(fr + Fraction(1, 2))


def sat(v, bits):
    return max(-(1 << (bits - 1)), min((1 << (bits - 1)) - 1, v))


# ---------------------------------------------------------------- rhu / rsh_r
def test_rhu_against_rationals(orc):
    for d in list(range(1, 40)) + [255, 256, 257, 4096, 32767, 2**25 - 1]:
        for n in list(range(-200, 201)) + [10**9 + 7, -(10**9) - 7, 2**40 + 1, -(2**40) - 1]:
            assert orc.rhu(n, d) == exact_round_half_up(Fraction(n, d)), (n, d)


def test_rsh_r_against_rationals(orc):
    rnd = random.Random(1)
    for k in range(1, 40):
        vals = list(range(-70, 71)) + [rnd.randrange(-2**50, 2**50) for _ in range(50)]
        for a in vals:
            assert orc.rsh_r(a, k) == exact_round_half_up(Fraction(a, 1 << k)), (a, k)


# ---------------------------------------------------------------- rescale
def test_rescale_exhaustive_small_range(orc):
    """All a in [-4096, 4096] x e in [-24, 4] x several M, against the exact
    rational floor(a * M * 2^(e-31) + 1/2)."""
    rnd = random.Random(2)
    Ms = [2**30, 2**30 + 1, 2**31 - 1] + [rnd.randrange(2**30, 2**31) for _ in range(5)]
    for M in Ms:
        for e in range(-24, 5):
            scale = Fraction(M, 1 << (31 - e))
            for a in range(-4096, 4097, 1 if M in Ms[:3] and e % 4 == 0 else 37):
                want = sat(exact_round_half_up(a * scale), 32)
                assert orc.rescale(a, M, e) == want, (a, M, e)


def test_rescale_random_full_range(orc):
    rnd = random.Random(3)
    for _ in range(20000):
        a = rnd.randrange(-2**31, 2**31)
        M = rnd.randrange(2**30, 2**31)
        e = rnd.randrange(-31, 31)
        want = sat(exact_round_half_up(Fraction(a * M, 1 << (31 - e))), 32)
        assert orc.rescale(a, M, e) == want, (a, M, e)


def test_rescale_ties_round_up_and_saturation(orc):
    M, e = 2**30, 0  # scale exactly 1/2
    assert orc.rescale(1, M, e) == 1  # 0.5 -> 1
    assert orc.rescale(-1, M, e) == 0  # -0.5 -> 0 (ties toward +inf)
    assert orc.rescale(-3, M, e) == -1  # -1.5 -> -1
    M, e = 2**31 - 1, 30  # scale just below 2^30
    assert orc.rescale(2**31 - 1, M, e) == 2**31 - 1
    assert orc.rescale(-(2**31), M, e) == -(2**31)
    assert orc.rescale(4, 2**30, 30) == 2**31 - 1  # 4 * 2^29 = 2^31 saturates
    assert orc.rescale(-4, 2**30, 30) == -(2**31)


# ---------------------------------------------------------------- quantize_multiplier
def test_quantize_multiplier_properties(orc):
    rnd = random.Random(4)
    for _ in range(5000):
        s = math.ldexp(rnd.uniform(0.5, 1.0), rnd.randrange(-30, 30))
        M, e = orc.quantize_multiplier(s)
        assert 2**30 <= M < 2**31
        assert abs(Fraction(M, 1 << 31) * Fraction(2) ** e / Fraction(s) - 1) <= Fraction(1, 2**31)
    for k in range(-31, 30):
        assert orc.quantize_multiplier(math.ldexp(1.0, k)) == (2**30, k + 1)
    # a mantissa that rounds up to 2^31 is renormalized
    M, e = orc.quantize_multiplier(1.0 - 2.0**-40)
    assert (M, e) == (2**30, 1)


def test_quantize_multiplier_rejects(orc):
    for bad in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(orc.OracleError) as ei:
            orc.quantize_multiplier(bad)
        assert ei.value.code == orc.BAD_RANGE
    for s in (2.0**-33, 2.0**31):
        with pytest.raises(orc.OracleError) as ei:
            orc.quantize_multiplier(s)
        assert ei.value.code == orc.UNSUPPORTED


# ---------------------------------------------------------------- isqrt
def test_isqrt_defining_inequality(orc):
    for v in range(0, 1 << 14):
        r = orc.isqrt(v)
        assert r * r <= v < (r + 1) * (r + 1)
    rnd = random.Random(5)
    for _ in range(20000):
        v = rnd.randrange(0, 2**62)
        r = orc.isqrt(v)
        assert r * r <= v < (r + 1) * (r + 1)
    for r in (2**25, 2**31 - 1, 3037000499):
        assert orc.isqrt(r * r) == r and orc.isqrt(r * r - 1) == r - 1


# ---------------------------------------------------------------- sigmoid / tanh
def test_expneg_against_libm(orc):
    for y in list(range(0, 1 << 16, 7)) + [2**20 - 1, 2**20, 2**24]:
        got = orc.expneg(y) / 2.0**31
        want = math.exp(-min(y, 2**20 - 1) / 2.0**15)
        assert abs(got - want) < 2.0**-20, y


@pytest.mark.parametrize("m", range(0, 9))
def test_sigmoid_tanh_exhaustive_against_libm(orc, m):
    """All 65536 inputs of each format: within 0.51 LSB of the real function
    away from the output clamp, within 1 LSB at it; monotone; mirrored."""
    prev_s, prev_t = -1, -32769
    for x in range(-32768, 32768):
        r = x / 2.0 ** (15 - m)
        s, t = orc.int_sigmoid(x, m), orc.int_tanh(x, m)
        fs, ft = 32768.0 / (1.0 + math.exp(-r)), 32768.0 * math.tanh(r)
        assert 0 <= s <= GOLD["activation_output_clamp"]["hi"]
        assert GOLD["activation_output_clamp"]["lo"] <= t <= GOLD["activation_output_clamp"]["hi"]
        assert abs(s - fs) <= (0.51 if s < 32767 else 1.0), (x, m)
        assert abs(t - ft) <= (0.51 if abs(t) < 32767 else 1.0), (x, m)
        assert s >= prev_s and t >= prev_t, (x, m)
        prev_s, prev_t = s, t
    for x in range(1, 32768, 13):
        # sigma(x) + sigma(-x) = 1 and tanh odd, up to the output clamp
        sp, sn = orc.int_sigmoid(x, m), orc.int_sigmoid(-x, m)
        assert sp + sn == 32768 or (sp == 32767 and sn == 0)
        tp, tn = orc.int_tanh(x, m), orc.int_tanh(-x, m)
        assert tp == -tn or (tp == 32767 and tn == -32768)


def test_activation_values_the_paper_prints(orc):
    # 1 - tanh(8) = 2.35e-7 is far below half an LSB of Q0.15: the top of Q3.12
    # maps to the top of the clamped output range.
    assert 1.0 - math.tanh(8.0) == pytest.approx(GOLD["tanh_clamp_error_at_8"]["value"], rel=0.05)
    assert orc.int_tanh(32767, 3) == 32767
    assert orc.int_tanh(-32768, 3) == -32768
    # one Q3.12 step at the origin moves tanh by tanh(2^-12) = 2.44e-4 = 8 LSB of Q0.15
    assert math.tanh(2.0**-12) == pytest.approx(GOLD["tanh_resolution_q3_12"]["value"], rel=0.01)
    assert orc.int_tanh(1, 3) == round(GOLD["tanh_resolution_q3_12"]["value"] * 32768) == 8
    assert orc.int_sigmoid(0, 3) == 16384 and orc.int_tanh(0, 3) == 0
    assert orc.int_tanh(4096, 3) == round(math.tanh(1.0) * 32768)
    assert orc.int_sigmoid(4096, 3) == round(32768 / (1 + math.exp(-1.0)))
    assert orc.int_sigmoid(32767, 3) == round(32768 / (1 + math.exp(-32767 / 4096.0)))
    assert orc.int_sigmoid(-32768, 3) == round(32768 / (1 + math.exp(8.0)))
    assert orc.int_sigmoid(32767, 6) == 32767 and orc.int_sigmoid(-32768, 6) == 0


# ---------------------------------------------------------------- layer norm
def _float_layernorm(q, L, b):
    q = q.astype(np.float64)
    mean, sd = q.mean(), q.std()
    return (q - mean) / sd * L + b


@pytest.mark.parametrize("n", [2, 64, 512, 2048, 4096])
def test_layernorm_against_double(orc, n):
    rng = np.random.default_rng(n)
    for trial in range(6):
        spread = [30000, 8000, 500, 20, 3, 10000][trial]
        q = np.clip(rng.normal(rng.integers(-2000, 2000), spread, size=n), -32767, 32767).astype(np.int16)
        if q.std() == 0:
            continue
        L = rng.uniform(0.5, 1.5, size=n)
        b = rng.uniform(-0.1, 0.1, size=n)
        sL = np.abs(L).max() / 32767.0
        qL = np.floor(L / sL + 0.5).astype(np.int16)
        qb = np.floor(b / (sL * 2.0**-10) + 0.5).astype(np.int32)
        M, e = orc.quantize_multiplier(sL * 4096.0)
        out = orc.int_layernorm(q, qL, qb, M, e)
        want = _float_layernorm(q, qL * sL, qb * sL * 2.0**-10)
        # one Q3.12 LSB of output rounding + the 2^-10 resolution of x' times
        # |L| + the relative error of the floored sigma (1/sigma, sigma = 2^10 sd)
        tol = 1.0 + 4096.0 * (1.5 * 2.0**-10) + 4096.0 * np.abs(want) / (1024.0 * q.std())
        got = out.astype(np.float64)
        ok = np.abs(np.clip(want * 4096.0, -32768, 32767) - got) <= tol + 0.51
        assert ok.all(), (n, trial, np.abs(want * 4096 - got).max())


def test_layernorm_invariants(orc):
    rng = np.random.default_rng(7)
    n = 1024
    q = rng.normal(0, 3000, size=n).astype(np.int16)
    qL = np.full(n, 32767, dtype=np.int16)  # L = 1 exactly at s_L = 1/32767
    qb = np.zeros(n, dtype=np.int32)
    M, e = orc.quantize_multiplier(4096.0 / 32767.0)
    out = orc.int_layernorm(q, qL, qb, M, e).astype(np.float64) / 4096.0
    assert abs(out.mean()) < 2e-3 and abs((out**2).mean() - 1.0) < 5e-3
    # any scale of the input cancels (Sec. 3.2.6): doubling q changes nothing
    # beyond rounding
    out2 = orc.int_layernorm((q // 2 * 2).astype(np.int16), qL, qb, M, e).astype(np.float64)
    out1 = orc.int_layernorm((q // 2).astype(np.int16), qL, qb, M, e).astype(np.float64)
    assert np.abs(out2 - out1).max() <= 6
    # constant row: sigma = 0 -> only the bias survives
    qb = rng.integers(-2**20, 2**20, size=n).astype(np.int32)
    outc = orc.int_layernorm(np.full(n, 1234, dtype=np.int16), qL, qb, M, e)
    want = [sat(orc.rescale(sat(orc.rsh_r(int(v), 10), 32), M, e), 16) for v in qb]
    assert outc.tolist() == want
    # n = 1 is a constant row
    assert orc.int_layernorm(np.array([77], np.int16), qL[:1], qb[:1], M, e).tolist() == want[:1]


def test_layernorm_extra_factor_restores_resolution(orc):
    """Sec. 3.2.6: x' alone spans about 2.8 bits; with s' = 2^-10 the
    normalized integers q' = x' / s' carry 10 more.  The output resolution of
    the integer path must therefore be far better than 1/8 (3 bits)."""
    assert GOLD["layernorm_extra_factor"]["log2"] == -10
    rng = np.random.default_rng(11)
    n = 2048
    q = rng.normal(0, 4000, size=n).astype(np.int16)
    qL = np.full(n, 32767, dtype=np.int16)
    qb = np.zeros(n, dtype=np.int32)
    M, e = orc.quantize_multiplier(4096.0 / 32767.0)
    out = orc.int_layernorm(q, qL, qb, M, e).astype(np.float64) / 4096.0
    want = _float_layernorm(q, np.ones(n), np.zeros(n))
    assert np.abs(out - want).max() < 2.0**-8
    assert len(np.unique(out)) > 1000  # not a 2.8-bit staircase


def test_layernorm_limits(orc):
    with pytest.raises(orc.OracleError):
        orc.int_layernorm(np.zeros(4097, np.int16), np.zeros(4097, np.int16), np.zeros(4097, np.int32),
                          2**30, 0)
    # the largest row at the extreme values stays inside int64 (exact sums)
    n = 4096
    q = np.full(n, -32768, dtype=np.int16)
    q[::2] = 32767
    qL = np.full(n, -32767, dtype=np.int16)
    qb = np.full(n, 2**31 - 1, dtype=np.int32)
    M, e = orc.quantize_multiplier(0.1875)
    out = orc.int_layernorm(q, qL, qb, M, e)
    mean = exact_round_half_up(Fraction(int(q.astype(np.int64).sum()) * 1024, n))
    var = exact_round_half_up(Fraction(int((q.astype(np.int64) ** 2).sum()) << 20, n)) - mean * mean
    sigma = math.isqrt(var)
    for i in (0, 1, n - 1):
        qn = exact_round_half_up(Fraction(1024 * (1024 * int(q[i]) - mean), sigma))
        t = qn * int(qL[i]) + int(qb[i])
        q2 = sat(exact_round_half_up(Fraction(t, 1024)), 32)
        assert out[i] == sat(exact_round_half_up(Fraction(q2 * M, 1 << (31 - e))), 16)
