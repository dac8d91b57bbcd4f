"""Pins for the oracle's fp16 component format (App. A Table 7: 5 exponent bits, 10 stored
significand bits, machine epsilon 2^-10).

The chain code (Fast2Sum, Grow, Mul, the AdamW step) is the same template the bf16 pins cover; what is
new for fp16 is the decode W, the roundings R (from fp32) and B (from fp64), and the range.  They are
pinned here to exact rational arithmetic (fractions.Fraction over the table of all fp16 values), to
numpy's own IEEE binary16 type (an implementation this repository did not write), to the exactness
properties of the error-free transformations, to hand-computed scalar patterns and to a textbook fp64
AdamW.
"""
import bisect
from fractions import Fraction

import numpy as np
import pytest

F16 = 1          # oracle format id
rng = np.random.default_rng(20240516)


def f16_fraction(h):
    """Exact value of a finite binary16 pattern, from the format's definition."""
    h = int(h)
    sign = -1 if h & 0x8000 else 1
    e, mant = (h >> 10) & 0x1F, h & 0x3FF
    assert e != 31
    if e == 0:
        return sign * Fraction(mant, 2 ** 24)
    return sign * Fraction(1024 + mant) * Fraction(2) ** (e - 25)


_POS = [f16_fraction(h) for h in range(0, 0x7C00)]
_OVER = _POS[-1] + (_POS[-1] - _POS[-2]) / 2


def nearest_f16(x):
    x = Fraction(x)
    sign = 0x8000 if x < 0 else 0
    a = abs(x)
    if a >= _OVER:
        return sign | 0x7C00
    i = bisect.bisect_right(_POS, a) - 1
    if _POS[i] == a or i == 0x7BFF:
        return sign | i
    dlo, dhi = a - _POS[i], _POS[i + 1] - a
    if dlo != dhi:
        return sign | (i if dlo < dhi else i + 1)
    return sign | (i if i % 2 == 0 else i + 1)


def ulp16(x):
    a = abs(Fraction(x))
    e = -14
    if a >= Fraction(1, 2 ** 14):
        e = 15
        while Fraction(2) ** e > a:
            e -= 1
    return Fraction(2) ** (max(e, -14) - 10)


def as_f64(u):
    return np.asarray(u, np.uint16).view(np.float16).astype(np.float64)


def finite_patterns(n, lo_exp=0, hi_exp=30, signed=True):
    """Random finite fp16 patterns with exponent field in [lo_exp, hi_exp]."""
    e = rng.integers(lo_exp, hi_exp + 1, n).astype(np.uint16)
    m = rng.integers(0, 1024, n).astype(np.uint16)
    s = (rng.integers(0, 2, n).astype(np.uint16) << 15) if signed else np.uint16(0)
    return (s | (e << 10) | m).astype(np.uint16)


# ---- W, R, B ---------------------------------------------------------------------------------
def test_widen_every_pattern(orc):
    h = np.arange(65536, dtype=np.uint16)
    got = orc.widen_array(h, fmt=F16)
    want = h.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))      # signs of zero included
    for p in (0x0001, 0x03FF, 0x0400, 0x3C00, 0x3C01, 0x7BFF, 0x8001, 0xC000):
        assert Fraction(orc.widen(p, fmt=F16)) == f16_fraction(p)


def test_R_fixed_points_midpoints_and_random_fp32(orc):
    pos = np.arange(0x7C00, dtype=np.uint16)
    vals = pos.view(np.float16).astype(np.float32)
    assert np.array_equal(orc.R_array(vals, fmt=F16), pos)                      # every fp16 value is a fixed point
    assert np.array_equal(orc.R_array(-vals, fmt=F16), pos | 0x8000)
    mid = ((vals[:-1].astype(np.float64) + vals[1:].astype(np.float64)) / 2).astype(np.float32)   # exact in fp32
    even = np.where(pos[:-1] % 2 == 0, pos[:-1], pos[1:])
    assert np.array_equal(orc.R_array(mid, fmt=F16), even)                      # ties go to the even pattern
    up = np.nextafter(mid, np.float32(np.inf))
    dn = np.nextafter(mid, np.float32(0))
    assert np.array_equal(orc.R_array(up, fmt=F16), pos[1:])
    assert np.array_equal(orc.R_array(dn, fmt=F16), pos[:-1])
    # overflow rule: the midpoint between the largest finite value and 2^16 goes to infinity
    assert orc.R(65519.996, fmt=F16) == 0x7BFF and orc.R(65520.0, fmt=F16) == 0x7C00
    assert orc.R(float("inf"), fmt=F16) == 0x7C00 and orc.R(-float("inf"), fmt=F16) == 0xFC00
    assert orc.R(float("nan"), fmt=F16) == 0x7E00
    assert orc.R(-0.0, fmt=F16) == 0x8000
    bits = rng.integers(0, 2 ** 32, 1 << 20, dtype=np.uint64).astype(np.uint32)
    f = bits.view(np.float32)
    with np.errstate(over="ignore"):
        want = f.astype(np.float16).view(np.uint16)
    got = orc.R_array(f, fmt=F16)
    nan = np.isnan(f)
    assert np.array_equal(got[~nan], want[~nan]) and np.all(got[nan] == 0x7E00)


def test_B_is_a_single_rounding(orc):
    # just above a tie in fp64 but ON the tie once rounded to fp32: a detour through fp32 would give the
    # even neighbour, one rounding gives the upper one
    for lo in (0x3C00, 0x3C02, 0x0400, 0x0002, 0x7BFE, 0x5640):
        a, b = f16_fraction(lo), f16_fraction(lo + 1)
        x = float((a + b) / 2) * (1 + 2.0 ** -40)
        assert np.float32(x) == np.float32(float((a + b) / 2))
        assert orc.B(x, fmt=F16) == lo + 1 == nearest_f16(Fraction(x))
        assert orc.B(-x, fmt=F16) == (lo + 1) | 0x8000
    xs = np.concatenate([rng.normal(0, 1, 4000) * 10.0 ** rng.integers(-9, 6, 4000), [0.0, 2.0 ** -25, 2.0 ** -24, 65519.99, 65520.0, 1e9]])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).view(np.uint16)           # numpy converts fp64 -> fp16 directly
    for x, w in zip(xs[:1500], want[:1500]):
        assert orc.B(x, fmt=F16) == int(w) == nearest_f16(Fraction(float(x)))
    for x, w in zip(xs[1500:], want[1500:]):
        assert orc.B(x, fmt=F16) == int(w)
    assert orc.B(2.0 ** -25, fmt=F16) == 0 and orc.B(2.0 ** -25 * 1.0000001, fmt=F16) == 1     # half the least subnormal: tie to even


# ---- F(a o b) --------------------------------------------------------------------------------
@pytest.mark.parametrize("op", [0, 1, 2, 3])
def test_binop_is_the_correctly_rounded_exact_result(orc, op):
    n = 3000
    a = np.concatenate([finite_patterns(n), finite_patterns(400, 0, 2), finite_patterns(400, 28, 30)])
    b = np.concatenate([finite_patterns(n), finite_patterns(400, 0, 2), finite_patterns(400, 28, 30)])[::-1].copy()
    if op == 3:
        b[(b & 0x7FFF) == 0] = 0x3C00
    got = orc.binop(op, a, b, fmt=F16)
    for x, y, g in zip(a, b, got):
        fx, fy = f16_fraction(x), f16_fraction(y)
        exact = (fx + fy, fx - fy, fx * fy, fx / fy if fy else None)[op]
        want = nearest_f16(exact)
        if exact == 0:                                    # sign of an exact zero follows IEEE, not the rational
            assert g & 0x7FFF == 0
        else:
            assert g == want, (hex(x), hex(y), hex(g), hex(want))


def test_binops_against_numpy_half_arithmetic(orc):
    n = 1 << 20
    a, b = finite_patterns(n), finite_patterns(n)
    fa, fb = a.view(np.float16), b.view(np.float16)
    with np.errstate(all="ignore"):
        wants = [fa + fb, fa - fb, fa * fb, fa / fb, np.sqrt(fa)]
    for op, w in enumerate(wants):
        got = orc.binop(op, a, b, fmt=F16)
        nan = np.isnan(w)
        assert np.array_equal(got[~nan], w.view(np.uint16)[~nan]), op
        assert np.all(got[nan] == 0x7E00), op


def test_sqrt_brackets_the_exact_root(orc):
    a = finite_patterns(4000, signed=False)
    got = orc.binop(4, a, fmt=F16)
    for x, g in zip(a, got):
        fx, r = f16_fraction(x), f16_fraction(g)
        if fx == 0:
            assert r == 0
            continue
        lo = (r + f16_fraction(g - 1)) / 2 if g else Fraction(0)
        hi = (r + f16_fraction(g + 1)) / 2
        assert lo * lo <= fx <= hi * hi, hex(x)


# ---- error-free transformations --------------------------------------------------------------
def test_fast2sum_and_two_sum_are_exact(orc):
    n = 20000
    a, b = finite_patterns(n, 0, 29), finite_patterns(n, 0, 29)          # below 2^15: no overflow
    big = np.abs(as_f64(a)) >= np.abs(as_f64(b))
    hi, lo = np.where(big, a, b), np.where(big, b, a)
    x, y = orc.fast2sum(hi, lo, fmt=F16)
    assert np.array_equal(as_f64(x) + as_f64(y), as_f64(hi) + as_f64(lo))        # fp64 holds these sums exactly
    x2, y2 = orc.two_sum(a, b, fmt=F16)                                           # any order
    assert np.array_equal(as_f64(x2) + as_f64(y2), as_f64(a) + as_f64(b))
    assert np.array_equal(x2, x)
    same = as_f64(y2) == as_f64(y)
    assert same.all()
    for i in range(300):                                   # non-overlap: |y| <= ulp(x)/2
        assert abs(f16_fraction(y[i])) <= ulp16(f16_fraction(x[i])) / 2


def test_fast2sum_loses_the_error_when_unsorted_and_two_sum_does_not(orc):
    a, b = np.array([0x1400], np.uint16), np.array([0x3C01], np.uint16)      # 2^-10 and 1+2^-10, |a| < |b|
    x, y = orc.fast2sum(a, b, fmt=F16)
    x2, y2 = orc.two_sum(a, b, fmt=F16)
    exact = f16_fraction(a[0]) + f16_fraction(b[0])
    assert f16_fraction(x2[0]) + f16_fraction(y2[0]) == exact
    assert x[0] == x2[0]


def test_two_prod_fma_is_exact_in_range(orc):
    n = 20000
    a, b = finite_patterns(n, 13, 19), finite_patterns(n, 13, 19)        # |.| in [2^-2, 2^5): product error >= 2^-24
    x, e = orc.two_prod_fma(a, b, fmt=F16)
    assert np.array_equal(as_f64(x) + as_f64(e), as_f64(a) * as_f64(b))
    assert np.array_equal(x, orc.binop(2, a, b, fmt=F16))


def test_grow_value_and_non_overlap(orc):
    n = 5000
    x = finite_patterns(n, 14, 18)                                        # |x| >= 0.5: ulp(x)/2 >= 2^-12
    y0 = finite_patterns(n, 0, 2)                                         # |y| < 2^-12: a valid second component
    a = finite_patterns(n, 3, 14)
    ok = np.abs(as_f64(x)) >= np.abs(as_f64(a))
    x, y0, a = x[ok], y0[ok], a[ok]
    gx, gy = orc.grow(x, y0, a, fmt=F16)
    exact = as_f64(x) + as_f64(y0) + as_f64(a)
    got = as_f64(gx) + as_f64(gy)
    assert np.all(np.abs(got - exact) <= 2.0 ** -20 * np.abs(exact) + 2.0 ** -24)     # second-order in 2^-11
    for i in range(400):
        assert abs(f16_fraction(gy[i])) <= ulp16(f16_fraction(gx[i])) / 2
    tx, ty = orc.grow_two_sum(x, y0, a, fmt=F16)
    assert np.array_equal(as_f64(tx) + as_f64(ty), got)


def test_mul_and_scaling_relative_error(orc):
    n = 5000
    a1, b1 = finite_patterns(n, 14, 17), finite_patterns(n, 14, 17)
    a2 = orc.binop(2, a1, np.full(n, 0x0E00, np.uint16), fmt=F16)        # about 2^-12 * a1, within half an ulp
    b2 = orc.binop(2, b1, np.full(n, 0x8D00, np.uint16), fmt=F16)
    x, e = orc.mul_expansion(a1, a2, b1, b2, fmt=F16)
    exact = (as_f64(a1) + as_f64(a2)) * (as_f64(b1) + as_f64(b2))
    assert np.all(np.abs(as_f64(x) + as_f64(e) - exact) <= 2.0 ** -18 * np.abs(exact))
    one = np.abs(as_f64(x) - exact) / np.abs(exact)
    assert one.max() > 2.0 ** -13                                          # a single fp16 could not do that
    sx, se = orc.scaling(b1, a1, a2, fmt=F16)
    exact = as_f64(b1) * (as_f64(a1) + as_f64(a2))
    assert np.all(np.abs(as_f64(sx) + as_f64(se) - exact) <= 2.0 ** -18 * np.abs(exact))


# ---- scalars and the step ----------------------------------------------------------------------
def test_scalar_patterns_by_hand(orc):
    s = orc.scalars(1e-3, 0.9, 0.999, 1e-8, 0.1, 1, fmt=F16)
    # 0.999 lies between 2045/2048 and 2046/2048, nearer the latter: exponent field 14, significand 1022
    assert s["b2"] == (14 << 10) | 1022 == 0x3BFE
    # the second component is 0.999 - 2046/2048 = -2.34375e-5 = -393.2 * 2^-24: a subnormal with 393 steps
    assert s["b2l"] == 0x8000 | 393
    assert s["b1"] == nearest_f16(Fraction(0.9)) and s["c1"] == nearest_f16(1 - Fraction(0.9))
    assert s["c2"] == nearest_f16(1 - Fraction(0.999))
    assert s["bc1"] == s["c1"] and s["bc2"] == s["c2"]                    # t = 1
    assert s["e"] == 0                                                     # 1e-8 is below half the least subnormal 2^-25
    assert s["na"] == nearest_f16(-Fraction(1e-3)) and s["lam"] == nearest_f16(Fraction(0.1))
    s7 = orc.scalars(1e-3, 0.9, 0.999, 1e-4, 0.1, 7, fmt=F16)
    assert s7["bc1"] == nearest_f16(1 - Fraction(0.9) ** 7) and s7["bc2"] == nearest_f16(1 - Fraction(0.999) ** 7)
    assert s7["e"] == nearest_f16(Fraction(1e-4))


def _to16(x):
    return np.asarray(x, np.float64).astype(np.float16).view(np.uint16).copy()


def _textbook(theta, m, v, g, hyper, t):
    lr, b1, b2, eps, wd = hyper
    m = b1 * m + (1 - b1) * g
    v = b2 * v + (1 - b2) * g * g
    mh, vh = m / (1 - b1 ** t), v / (1 - b2 ** t)
    return theta - lr * (mh / (np.sqrt(vh) + eps) + wd * theta), m, v


@pytest.mark.parametrize("variant", [0, 1])
def test_step_tracks_textbook_adamw_in_fp64(orc, variant):
    n, steps = 4096, 200
    hyper = (2e-4, 0.9, 0.98, 1e-4, 0.1)
    th64 = rng.normal(0, 1.0, n)
    th64 = as_f64(_to16(th64))
    theta, dth, m, v, dv = _to16(th64), _to16(np.zeros(n)), _to16(np.zeros(n)), _to16(np.zeros(n)), _to16(np.zeros(n))
    plain, pm, pv = theta.copy(), m.copy(), v.copy()
    m64, v64 = np.zeros(n), np.zeros(n)
    for t in range(1, steps + 1):
        g = _to16(rng.normal(0, 0.3, n))                          # g^2 stays far above the fp16 subnormals
        orc.adamw_step(theta, dth, m, v, dv if variant == 1 else None, g, variant | orc.STEP_FP16, hyper, t)
        orc.adamw_step(plain, None, pm, pv, None, g, orc.BF16 | orc.STEP_FP16, hyper, t)
        th64, m64, v64 = _textbook(th64, m64, v64, as_f64(g), hyper, t)
    err_mcf = np.abs(as_f64(theta) + as_f64(dth) - th64)
    err_plain = np.abs(as_f64(plain) - th64)
    assert np.isfinite(err_mcf).all()
    # 200 updates of about 2e-4 on parameters of order 1 (ulp 2^-10): the expansion follows fp64 to a
    # fraction of the total movement, a single fp16 loses most updates outright
    assert np.median(err_mcf) < 4e-4 and np.median(err_plain) > 5 * np.median(err_mcf)
    assert np.abs(as_f64(m) - m64).max() < 3e-3
    assert np.all(np.abs(as_f64(v) + (as_f64(dv) if variant == 1 else 0) - v64) <= 0.02 * v64 + 1e-6)


def test_first_step_by_hand(orc):
    # one element, values chosen so that every intermediate is exact or has an obvious rounding
    hyper = (0.5, 0.5, 0.5, 0.0, 0.0)
    theta, dth, m, v = _to16([1.0]), _to16([0.0]), _to16([0.0]), _to16([0.0])
    g = _to16([0.25])
    delta = np.zeros(1, np.uint16)
    orc.adamw_step(theta, dth, m, v, None, g, orc.LIGHT | orc.STEP_FP16, hyper, 1, delta_out=delta)
    # m = 0.125, v = 0.03125, bias corrections 0.5: m_hat = 0.25, v_hat = 0.0625, root 0.25, ratio 1, delta = -0.5
    assert as_f64(m)[0] == 0.125 and as_f64(v)[0] == 0.03125
    assert as_f64(delta)[0] == -0.5 and as_f64(theta)[0] == 0.5 and as_f64(dth)[0] == 0.0
    # a tiny update that one fp16 parameter would lose is kept in the second component
    hyper = (2.0 ** -13, 0.5, 0.5, 0.0, 0.0)
    theta, dth, m, v = _to16([1.0]), _to16([0.0]), _to16([0.0]), _to16([0.0])
    orc.adamw_step(theta, dth, m, v, None, g, orc.LIGHT | orc.STEP_FP16, hyper, 1)
    assert as_f64(theta)[0] == 1.0 and as_f64(dth)[0] == -(2.0 ** -13)
    plain = _to16([1.0])
    orc.adamw_step(plain, None, _to16([0.0]), _to16([0.0]), None, g, orc.BF16 | orc.STEP_FP16, hyper, 1)
    assert as_f64(plain)[0] == 1.0                                  # lost arithmetic (Def. 3.2)


def test_edq_in_fp16(orc):
    n = 1000
    th0, dth0 = finite_patterns(n, 14, 16), finite_patterns(n, 0, 2)
    delta = finite_patterns(n, 0, 5)
    th1, dth1 = orc.grow(th0, dth0, delta, fmt=F16)
    acc = orc.EdqAccumulator(fmt=F16)
    acc.add(delta, th0, dth0, th1, dth1)
    d = as_f64(delta)
    eff = (as_f64(th1) + as_f64(dth1)) - (as_f64(th0) + as_f64(dth0))
    want = float(np.dot(d, eff) / np.sqrt(np.dot(d, d)))
    assert abs(acc.value() - want) <= 1e-12 * abs(want)
    assert acc.lost.value == int(np.sum((d != 0) & (eff == 0)))
    plain = orc.binop(0, th0, delta, fmt=F16)
    lost = orc.EdqAccumulator(fmt=F16)
    lost.add(delta, th0, None, plain, None)
    assert lost.lost.value == int(np.sum(plain == th0)) > n // 3       # many of these updates vanish in one fp16
    assert acc.lost.value < n // 50                                    # the expansion keeps them
    assert abs(acc.value() - np.sqrt(np.dot(d, d))) <= 2e-3 * np.sqrt(np.dot(d, d))   # EDQ of an exact update is ||delta||


def test_bf16_and_fp16_steps_differ_only_through_the_format(orc):
    # the same call without the flag must be untouched by the format machinery
    n = 257
    hyper = (1e-3, 0.9, 0.95, 1e-8, 0.1)
    th = rng.integers(0x3C00, 0x3F00, n).astype(np.uint16)
    g = rng.integers(0x3800, 0x3B00, n).astype(np.uint16)
    outs = []
    for flag in (0, orc.STEP_FP16):
        a, d, m, v = th.copy(), np.zeros(n, np.uint16), np.zeros(n, np.uint16), np.zeros(n, np.uint16)
        orc.adamw_step(a, d, m, v, None, g, flag, hyper, 1)
        outs.append((a, d, m, v))
    assert not np.array_equal(outs[0][2], outs[1][2])
    s = orc.scalars(*hyper, 1, fmt=F16)
    m16 = orc.binop(0, orc.binop(2, np.full(n, s["b1"], np.uint16), np.zeros(n, np.uint16), fmt=F16),
                    orc.binop(2, np.full(n, s["c1"], np.uint16), g, fmt=F16), fmt=F16)
    assert np.array_equal(outs[1][2], m16)
