"""The arithmetic the kernels run (csrc/lstm_int_math.h and the activation
tables of prepare.cpp), compiled for the host, against the oracle: the same
integers on exhaustive or adversarial ranges.  (The device build of the same
header is covered by the GPU parity tests.)"""
import ctypes as C
import os
import random

import numpy as np
import pytest

from paper_2101_05453_amd import build as libbuild


@pytest.fixture(scope="module")
def hm():
    if not os.path.exists(libbuild.HOSTMATH_LIB):
        libbuild.build_hostmath()
    L = C.CDLL(libbuild.HOSTMATH_LIB)
    L.hm_isqrt.restype = C.c_int64
    L.hm_isqrt.argtypes = [C.c_int64]
    for f in ("hm_rescale", "hm_rescale_hi"):
        getattr(L, f).restype = C.c_int32
        getattr(L, f).argtypes = [C.c_int32] * 3
    L.hm_layernorm.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    L.hm_sigmoid_table.argtypes = [C.c_int, C.c_void_p]
    L.hm_tanh_table.argtypes = [C.c_int, C.c_void_p]
    L.hm_sigmoid.argtypes = [C.c_void_p, C.c_int32]
    L.hm_tanh.argtypes = [C.c_void_p, C.c_int32]
    L.hm_layernorm2.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    L.hm_cell_update32.argtypes = [C.c_int32] * 5
    L.hm_rescale_sat16_pre.argtypes = [C.c_int32] * 3
    L.hm_rescale_sat16_pre.restype = C.c_int32
    L.hm_rescale_ge32.restype = C.c_int32
    L.hm_rescale_ge32.argtypes = [C.c_int32] * 3
    L.hm_cell_update.argtypes = [C.c_int32] * 5
    L.hm_hidden.argtypes = [C.c_int32] * 5
    return L


def test_rescale_forms(orc, hm):
    rnd = random.Random(0)
    for _ in range(40000):
        a = rnd.randrange(-2**31, 2**31)
        M = rnd.randrange(2**30, 2**31)
        e = rnd.randrange(-31, 31)
        want = orc.rescale(a, M, e)
        assert hm.hm_rescale(a, M, 31 - e) == want, (a, M, e)
        if 31 - e >= 33:
            assert hm.hm_rescale_hi(a, M, 31 - e) == want, (a, M, e)
    for M in (2**30, 2**31 - 1, 1518500250):
        for e in (-31, -2, -1, 0, 5, 30):
            for a in list(range(-300, 300)) + [2**31 - 1, -2**31]:
                assert hm.hm_rescale(a, M, 31 - e) == orc.rescale(a, M, e)
                if 31 - e >= 33:
                    assert hm.hm_rescale_hi(a, M, 31 - e) == orc.rescale(a, M, e)


def test_rescale_ge32(orc, hm):
    rnd = random.Random(9)
    for _ in range(40000):
        a = rnd.randrange(-2**31, 2**31)
        M = rnd.randrange(2**30, 2**31)
        e = rnd.randrange(-31, 0)  # r = 31 - e >= 32
        assert hm.hm_rescale_ge32(a, M, 31 - e) == orc.rescale(a, M, e), (a, M, e)
    for a in list(range(-5, 6)) + [2**31 - 1, -2**31, 2**30, -2**30]:
        for M in (2**30, 2**31 - 1, 2**30 + 1):
            assert hm.hm_rescale_ge32(a, M, 32) == orc.rescale(a, M, -1)


@pytest.mark.parametrize("m", range(0, 9))
def test_wide_tables_every_prefix(orc, hm, m):
    """The wide form of the tables (the same encoding over all 32768 entries, of which a
    kernel keeps a prefix in LDS, plus the tail part): for every prefix length a kernel
    may choose -- any multiple of 1024 beyond the point from which the choice is legal --
    the lookup returns the table's value for EVERY |x| in 0..32768."""
    hm.hm_compress_wide.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int), C.POINTER(C.c_int)]
    hm.hm_lut_wide_mag.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int32]
    for kind in ("sigmoid", "tanh"):
        tab = np.zeros(32769, np.uint16)
        getattr(hm, f"hm_{kind}_table")(m, tab.ctypes.data)
        blob = np.zeros(32768 + 8192 + 3072, np.uint8)
        has_tail, flat_from = C.c_int(), C.c_int()
        sh = hm.hm_compress_wide(tab.ctypes.data, blob.ctypes.data, C.byref(has_tail), C.byref(flat_from))
        F = flat_from.value
        assert all(tab[a] == tab[32768] for a in range(F, 32769)) and (F == 0 or tab[F - 1] != tab[32768])
        if sh < 0:
            continue
        if m == 3:
            assert has_tail.value == 1 and sh >= 5
        # legal prefixes: with the tail part any multiple of 1024 from 16384 on; without it the table must be
        # flat from the last kept entry on
        doms = [d for d in range(1024, 32769, 1024) if (has_tail.value and d >= 16384) or d - 1 >= F]
        assert doms, (kind, m)  # every format that compresses has a legal prefix
        probe = sorted(set(doms[:3] + doms[-2:] + doms[len(doms) // 2:len(doms) // 2 + 1]))
        for dom in probe:
            with_tail = int(bool(has_tail.value) and dom - 1 < F)
            for a in range(0, 32769):
                assert hm.hm_lut_wide_mag(blob.ctypes.data, sh, dom, with_tail, a) == int(tab[a]), (kind, m, dom, a)


def test_isqrt(orc, hm):
    rnd = random.Random(1)
    vals = list(range(0, 5000)) + [rnd.randrange(0, 2**50) for _ in range(20000)]
    vals += [r * r + d for r in (2**24, 2**25 - 1, 33554431) for d in (-1, 0, 1)]
    vals += [r * r + d for r in [rnd.randrange(1, 2**26) for _ in range(5000)] + [2**26 - 1] for d in (-1, 0, 1, 2)
             if r * r + d < 2**52]
    for v in vals:
        assert hm.hm_isqrt(v) == orc.isqrt(v), v


@pytest.mark.parametrize("m", range(0, 9))
def test_activation_tables_exhaustive(orc, hm, m):
    sig = np.zeros(32769, np.uint16)
    tnh = np.zeros(32769, np.uint16)
    hm.hm_sigmoid_table(m, sig.ctypes.data)
    hm.hm_tanh_table(m, tnh.ctypes.data)
    for x in range(-32768, 32768):
        assert hm.hm_sigmoid(sig.ctypes.data, x) == orc.int_sigmoid(x, m), (x, m)
        assert hm.hm_tanh(tnh.ctypes.data, x) == orc.int_tanh(x, m), (x, m)


def _ln_case(rng, n, kind):
    if kind == "normal":
        q = np.clip(rng.normal(rng.integers(-3000, 3000), rng.choice([3, 50, 2000, 12000]), size=n), -32767, 32767)
    elif kind == "extreme":
        q = rng.choice([-32767, 32767], size=n)
    elif kind == "spike":
        q = np.full(n, rng.integers(-32767, 32767))
        q[rng.integers(0, n)] += rng.choice([-1, 1, 2, 500])
        q = np.clip(q, -32767, 32767)
    elif kind == "threshold":  # sigma around 2^12, where the kernel switches between its two second-stage forms
        q = np.clip(np.rint(rng.normal(rng.choice([-32000, -5, 31000]), rng.choice([3.6, 4.0, 4.4]), size=n)), -32767, 32767)
    elif kind == "near_constant":
        q = np.full(n, rng.integers(-32000, 32000)) + rng.integers(0, 2, size=n)
    else:
        q = np.full(n, rng.integers(-32767, 32767))
    qL = rng.integers(-32767, 32768, size=n)
    qb = rng.integers(-2**31 + 1, 2**31, size=n)
    if kind in ("extreme", "threshold"):
        qL[:] = rng.choice([-32767, 32767], size=n)
        qb[:] = rng.choice([-2**31 + 1, 2**31 - 1], size=n)
    return q.astype(np.int16), qL.astype(np.int16), qb.astype(np.int32)


def test_layernorm_matches_oracle(orc, hm):
    rng = np.random.default_rng(5)
    hm.hm_ln_row_is_narrow.argtypes = [C.c_void_p, C.c_int32]
    forms = {0: 0, 1: 0}  # rows that took the second stage with / without the int32 clamp
    for trial in range(480):
        n = int(rng.choice([1, 2, 3, 17, 64, 512, 1000, 2048, 4096]))
        kind = ["normal", "extreme", "spike", "near_constant", "constant", "threshold"][trial % 6]
        q, qL, qb = _ln_case(rng, n, kind)
        forms[hm.hm_ln_row_is_narrow(q.ctypes.data, n)] += 1
        M, e = int(rng.integers(2**30, 2**31)), int(rng.integers(-24, 4))
        want = orc.int_layernorm(q, qL, qb, M, e)
        got = np.zeros(n, np.int16)
        hm.hm_layernorm(q.ctypes.data, n, qL.ctypes.data, qb.ctypes.data, M, 31 - e, got.ctypes.data)
        assert (got == want).all(), (trial, n, kind)
        if True:  # the per-row-prepared form used by the persistent kernel
            got2 = np.zeros(n, np.int16)
            hm.hm_layernorm2(q.ctypes.data, n, qL.ctypes.data, qb.ctypes.data, M, 31 - e, got2.ctypes.data)
            assert (got2 == want).all(), (trial, n, kind)
    assert forms[0] > 100 and forms[1] > 100, forms


def test_rescale_sat16_from_high_word(orc, hm):
    # sat16(rescale(a, M, r)) from one 32-bit high product, with the operand
    # shifted (and clamped) first when r < 33
    rnd = random.Random(11)
    edge = [-2**31, -2**31 + 1, -2**30 - 1, -2**30, -2**30 + 1, -65537, -32769, -32768, -2, -1, 0, 1, 2, 32767,
            32768, 65536, 2**30 - 1, 2**30, 2**30 + 1, 2**31 - 2, 2**31 - 1]
    for r in range(3, 63):
        e = 31 - r
        Ms = [2**30, 2**31 - 1, 2**30 + 1] + [rnd.randrange(2**30, 2**31) for _ in range(6)]
        for M in Ms:
            vals = edge + [rnd.randrange(-2**31, 2**31) for _ in range(40)]
            # values around the saturation and rounding boundaries of this scale
            for y in (-32769, -32768, -32767, -1, 0, 1, 32766, 32767, 32768):
                a0 = (2 * y + 1) * 2**r // (2 * M)
                vals += [a0 + d for d in (-2, -1, 0, 1, 2)]
            for a in vals:
                if not -2**31 <= a < 2**31:
                    continue
                want = max(-32768, min(32767, orc.rescale(a, M, e)))
                assert hm.hm_rescale_sat16_pre(a, M, r) == want, (a, M, r)


def test_cell_update_and_hidden(orc, hm):
    rnd = random.Random(3)
    edge = [-32768, -32767, -1, 0, 1, 32767]
    for m_c in range(0, 9):
        cases = [(i, z, f, c) for i in (0, 1, 32767) for z in edge for f in (0, 1, 32767) for c in edge]
        cases += [(rnd.randrange(0, 32768), rnd.randrange(-32768, 32768), rnd.randrange(0, 32768),
                   rnd.randrange(-32768, 32768)) for _ in range(3000)]
        for i, z, f, c in cases:
            want = max(-32768, min(32767, orc.rsh_r(i * z, 15 + m_c) + orc.rsh_r(f * c, 15)))
            assert hm.hm_cell_update(i, z, f, c, m_c) == want
            assert hm.hm_cell_update32(i, z, f, c, m_c) == want
    for _ in range(5000):
        o, tc = rnd.randrange(0, 32768), rnd.randrange(-32768, 32768)
        M, e, zp = rnd.randrange(2**30, 2**31), rnd.randrange(-26, -18), rnd.randrange(-128, 128)
        want = max(-128, min(127, orc.rescale(o * tc, M, e) + zp))
        assert hm.hm_hidden(o, tc, M, 31 - e, zp) == want
    for f in (0, 1, 16384, 32767):
        assert hm.hm_cifg(f) == min(32768 - f, 32767)


def test_sparse_operand_packing(hm):
    """The 2:4 compressed form of recurrent weight rows (sparse MFMA operands): unpacking every lane's
    values through its index bits, at the k positions the layout states, gives the row back; and the
    sparse dot product over that form equals the dense one."""
    rng = np.random.default_rng(11)
    hm.hm_sparse24_row_ok.argtypes = [C.c_void_p, C.c_int]
    hm.hm_sparse24_pack_lane.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    for K in (4, 7, 62, 64, 100, 128, 640, 1023):
        for kind in ("two", "mixed", "empty"):
            row = np.zeros(K, np.int8)
            for k0 in range(0, K, 4):
                width = min(4, K - k0)
                n = {"two": 2, "mixed": int(rng.integers(0, 3)), "empty": 0}[kind]
                pos = rng.choice(width, size=min(n, width, 2), replace=False)
                vals = rng.integers(-128, 128, size=len(pos))
                vals[vals == 0] = 5
                row[k0 + pos] = vals
            assert hm.hm_sparse24_row_ok(row.ctypes.data, K) == 1
            steps = (K + 63) // 64
            back = np.zeros(steps * 64, np.int8)
            hvec = rng.integers(-128, 128, size=steps * 64).astype(np.int64)
            dot = 0
            for q in range(steps):
                for a in range(2):
                    vals = np.zeros(16, np.int8)
                    idx = C.c_uint32(0)
                    hm.hm_sparse24_pack_lane(row.ctypes.data, K, q, a, vals.ctypes.data, C.byref(idx))
                    for j in range(8):
                        kb = 64 * q + (0 if j < 4 else 32) + 16 * a + 4 * (j % 4)
                        p0 = (idx.value >> (4 * j)) & 3
                        p1 = (idx.value >> (4 * j + 2)) & 3
                        assert p0 < p1, (K, q, a, j, idx.value)
                        for s, pp in ((0, p0), (1, p1)):
                            v = int(vals[2 * j + s])
                            assert back[kb + pp] == 0
                            back[kb + pp] = v
                            dot += v * int(hvec[kb + pp])
            assert (back[:K] == row).all() and not back[K:].any(), (K, kind)
            assert dot == int((row.astype(np.int64) * hvec[:K]).sum())
    # three nonzeros in one aligned group: not 2:4
    bad = np.zeros(64, np.int8)
    bad[[8, 9, 11]] = 1
    assert hm.hm_sparse24_row_ok(bad.ctypes.data, 64) == 0
    ok = np.zeros(64, np.int8)
    ok[[7, 8, 9, 12]] = 1  # spans two groups
    assert hm.hm_sparse24_row_ok(ok.ctypes.data, 64) == 1
