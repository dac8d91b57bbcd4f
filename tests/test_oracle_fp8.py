"""Pins for the oracle's two FP8 component formats (App. A Table 7: E5M2 and E4M3), the paper's
"direct extension to 8-bit" (Sec. 7).  The formats are small enough for exhaustive checks: every
pattern, every operand pair.

The chain code is the template the bf16 pins cover.  New are the decode W, the roundings R and B and
the range rules, pinned here to the formats' definitions written out with exact rationals, to torch's
own float8 types, to exhaustive exactness properties of the error-free transformations, and to scalar
patterns worked by hand.
"""
import bisect
from fractions import Fraction

import numpy as np
import pytest
import torch

E5M2, E4M3 = 2, 3
FMTS = [E5M2, E4M3]
rng = np.random.default_rng(8)


class Fmt:
    """The format from its definition: exponent bits, stored significand bits, bias, special patterns."""

    def __init__(self, fmt):
        self.fmt = fmt
        if fmt == E5M2:
            self.mbits, self.bias, self.emin = 2, 15, -14
            self.inf, self.nan = 0x7C, 0x7E
            self.max_bits = 0x7B
        else:
            self.mbits, self.bias, self.emin = 3, 7, -6
            self.inf, self.nan = None, 0x7F            # no infinities; one NaN pattern per sign
            self.max_bits = 0x7E
        self.pos = [self.value(h) for h in range(self.max_bits + 1)]
        gap = self.pos[-1] - self.pos[-2]
        self.over = self.pos[-1] + gap / 2             # the midpoint to the first value that does not exist

    def is_nan(self, h):
        h &= 0x7F
        return h > 0x7C if self.fmt == E5M2 else h == 0x7F

    def is_inf(self, h):
        return self.fmt == E5M2 and (h & 0x7F) == 0x7C

    def value(self, h):
        sign = -1 if h & 0x80 else 1
        e, m = (h & 0x7F) >> self.mbits, h & ((1 << self.mbits) - 1)
        if e == 0:
            return sign * Fraction(m, 1 << self.mbits) * Fraction(2) ** self.emin
        return sign * (1 + Fraction(m, 1 << self.mbits)) * Fraction(2) ** (e - self.bias)

    def nearest(self, x):
        """Round-to-nearest-even of the rational x; beyond the range: infinity (E5M2) or NaN (E4M3)."""
        x = Fraction(x)
        sign = 0x80 if x < 0 else 0
        a = abs(x)
        if a > self.over or (a == self.over and self.max_bits % 2 == 1):
            return (sign | self.inf) if self.inf is not None else self.nan
        i = bisect.bisect_right(self.pos, a) - 1
        if self.pos[i] == a or i == self.max_bits:
            return sign | i
        dlo, dhi = a - self.pos[i], self.pos[i + 1] - a
        if dlo != dhi:
            return sign | (i if dlo < dhi else i + 1)
        return sign | (i if i % 2 == 0 else i + 1)

    def finite(self):
        return [h for h in range(256) if not self.is_nan(h) and not self.is_inf(h)]

    def ulp(self, x):
        a = abs(Fraction(x))
        e = self.emin
        while Fraction(2) ** (e + 1) <= a:
            e += 1
        return Fraction(2) ** (e - self.mbits)


F = {f: Fmt(f) for f in FMTS}
ALL = np.arange(256, dtype=np.uint16)


def f64(orc, h, fmt):
    return orc.widen_array(np.asarray(h, np.uint16), fmt=fmt).astype(np.float64)


# ---- W, R, B -----------------------------------------------------------------------------------
@pytest.mark.parametrize("fmt", FMTS)
def test_decode_every_pattern(orc, fmt):
    f = F[fmt]
    got = orc.widen_array(ALL, fmt=fmt)
    tdt = torch.float8_e5m2 if fmt == E5M2 else torch.float8_e4m3fn
    ref = torch.arange(256, dtype=torch.int32).to(torch.uint8).view(tdt).float().numpy()
    for h in range(256):
        if f.is_nan(h):
            assert np.isnan(got[h]) and np.isnan(ref[h])
        elif f.is_inf(h):
            assert np.isinf(got[h]) and (got[h] < 0) == bool(h & 0x80) and got[h] == ref[h]
        else:
            assert Fraction(float(got[h])) == f.value(h), hex(h)
            assert got[h] == ref[h] and np.signbit(got[h]) == bool(h & 0x80)
    if fmt == E4M3:
        assert float(got[0x7E]) == 448.0 and float(got[0x01]) == 2.0 ** -9          # largest and smallest magnitudes
    else:
        assert float(got[0x7B]) == 57344.0 and float(got[0x01]) == 2.0 ** -16


@pytest.mark.parametrize("fmt", FMTS)
def test_R_fixed_points_ties_neighbours_and_range(orc, fmt):
    f = F[fmt]
    vals = np.array([float(v) for v in f.pos], np.float32)
    pos = np.arange(f.max_bits + 1, dtype=np.uint16)
    assert np.array_equal(orc.R_array(vals, fmt=fmt), pos)
    assert np.array_equal(orc.R_array(-vals, fmt=fmt), pos | 0x80)
    mid = ((vals[:-1].astype(np.float64) + vals[1:].astype(np.float64)) / 2).astype(np.float32)
    even = np.where(pos[:-1] % 2 == 0, pos[:-1], pos[1:])
    assert np.array_equal(orc.R_array(mid, fmt=fmt), even)
    assert np.array_equal(orc.R_array(np.nextafter(mid, np.float32(np.inf)), fmt=fmt), pos[1:])
    assert np.array_equal(orc.R_array(np.nextafter(mid, np.float32(0)), fmt=fmt), pos[:-1])
    top = float(f.over)
    beyond = (0x7C if fmt == E5M2 else 0x7F)
    below = np.nextafter(np.float32(top), np.float32(0))
    assert orc.R(float(below), fmt=fmt) == f.max_bits
    # the midpoint past the largest value: E5M2's largest has an odd significand, so the tie goes up to
    # infinity; E4M3's largest (0x7E) is even, so the tie stays, and only what lies above becomes NaN
    assert orc.R(top, fmt=fmt) == (0x7C if fmt == E5M2 else 0x7E)
    assert orc.R(float(np.nextafter(np.float32(top), np.float32(np.inf))), fmt=fmt) == beyond
    for big in (1e6, 3e38, float("inf")):
        assert orc.R(big, fmt=fmt) == beyond and orc.R(-big, fmt=fmt) == (0xFC if fmt == E5M2 else 0x7F)
    assert orc.R(float("nan"), fmt=fmt) == f.nan
    assert orc.R(-0.0, fmt=fmt) == 0x80 and orc.R(1e-30, fmt=fmt) == 0 and orc.R(-1e-30, fmt=fmt) == 0x80


@pytest.mark.parametrize("fmt", FMTS)
def test_R_random_fp32_against_the_definition(orc, fmt):
    f = F[fmt]
    bits = rng.integers(0, 2 ** 32, 1 << 18, dtype=np.uint64).astype(np.uint32)
    # half of the draws inside the format's own range so that most are not trivially zero or overflow
    lo_e, hi_e = (127 - 18, 127 + 17) if fmt == E5M2 else (127 - 11, 127 + 10)
    k = bits.size // 2
    bits[:k] = (bits[:k] & 0x807FFFFF) | (rng.integers(lo_e, hi_e, k).astype(np.uint32) << 23)
    x = bits.view(np.float32)
    got = orc.R_array(x, fmt=fmt)
    table = np.array([float(v) for v in f.pos])
    with np.errstate(invalid="ignore"):
        a = np.abs(x.astype(np.float64))
    fin = np.isfinite(a)
    i = np.clip(np.searchsorted(table, a, side="right") - 1, 0, f.max_bits)
    lo = table[i]
    hi = table[np.minimum(i + 1, f.max_bits)]
    dlo, dhi = a - lo, hi - a
    up = (dhi < dlo) | ((dhi == dlo) & (i % 2 == 1))
    want = np.where(up & (i < f.max_bits), i + 1, i).astype(np.uint16)
    over = float(f.over)
    beyond = np.uint16(0x7C if fmt == E5M2 else 0x7F)
    out_of_range = (a > over) | ((a == over) & (fmt == E5M2)) | ~fin
    want = np.where(out_of_range, beyond, want)
    sign = np.where(np.signbit(x), 0x80, 0).astype(np.uint16)
    want = np.where((want == 0x7F) & (fmt == E4M3), np.uint16(0x7F), want | sign)
    want = np.where(np.isnan(x), np.uint16(f.nan), want)
    bad = np.flatnonzero(got != want)
    assert bad.size == 0, (x[bad[:3]], got[bad[:3]], want[bad[:3]])
    for j in rng.integers(0, x.size, 300):                      # and the scalar rational search on a few
        if np.isfinite(x[j]):
            assert got[j] == f.nearest(Fraction(float(x[j])))


@pytest.mark.parametrize("fmt", FMTS)
def test_B_is_a_single_rounding(orc, fmt):
    f = F[fmt]
    for lo in (0x38, 0x39, 0x01, 0x10, 0x55, f.max_bits - 1):
        mid = float((f.pos[lo] + f.pos[lo + 1]) / 2)
        x = mid * (1 + 2.0 ** -40)                 # above the tie in fp64, on it once rounded to fp32
        assert np.float32(x) == np.float32(mid)
        assert orc.B(x, fmt=fmt) == lo + 1 == f.nearest(Fraction(x))
        assert orc.B(-x, fmt=fmt) == (lo + 1) | 0x80
    xs = np.concatenate([rng.normal(0, 1, 1500) * 10.0 ** rng.integers(-6, 4, 1500), [0.0, 0.95, 0.999, 3e-4, 1e-8, 0.1]])
    for x in xs:
        assert orc.B(float(x), fmt=fmt) == f.nearest(Fraction(float(x))), x


# ---- F(a o b): every operand pair ------------------------------------------------------------------
@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("op", [0, 1, 2, 3])
def test_binop_every_pair(orc, fmt, op):
    f = F[fmt]
    aa, bb = np.repeat(ALL, 256), np.tile(ALL, 256)
    got = orc.binop(op, aa, bb, fmt=fmt)
    wa, wb = f64(orc, ALL, fmt), f64(orc, ALL, fmt)
    fin = [h for h in range(256) if not f.is_nan(h) and not f.is_inf(h)]
    for a in fin:
        fa = f.value(a)
        for b in fin:
            fb = f.value(b)
            g = int(got[a * 256 + b])
            if op == 3 and fb == 0:
                # x/0: fp32 gives an infinity (NaN for 0/0); E5M2 keeps it, E4M3 has none and stores NaN
                if fa == 0 or fmt == E4M3:
                    assert f.is_nan(g)
                else:
                    assert f.is_inf(g) and bool(g & 0x80) == ((fa < 0) != bool(b & 0x80))
                continue
            exact = (fa + fb, fa - fb, fa * fb, None)[op] if op != 3 else fa / fb
            w = f.nearest(exact)
            if exact == 0:
                assert g & 0x7F == 0
            elif f.is_nan(w):
                assert f.is_nan(g)
            else:
                assert g == w, (hex(a), hex(b), hex(g), hex(w))
    # anything with a NaN operand is NaN, stored as the one pattern
    nan_rows = [h for h in range(256) if f.is_nan(h)]
    for a in nan_rows:
        assert np.all(got[a * 256:(a + 1) * 256] == f.nan)
    assert wa.shape == wb.shape


@pytest.mark.parametrize("fmt", FMTS)
def test_sqrt_every_pattern(orc, fmt):
    f = F[fmt]
    got = orc.binop(4, ALL, fmt=fmt)
    for h in range(256):
        g = int(got[h])
        if f.is_nan(h):
            assert g == f.nan
        elif f.is_inf(h):
            assert g == (0x7C if not h & 0x80 else f.nan)
        elif f.value(h) < 0:
            assert g == f.nan
        elif f.value(h) == 0:
            assert g == h                                           # sqrt(-0) = -0
        else:
            r = f.value(g)
            lo = (r + f.value(g - 1)) / 2
            hi = (r + f.value(g + 1)) / 2 if g < f.max_bits else f.over
            assert lo * lo <= f.value(h) <= hi * hi, hex(h)


# ---- error-free transformations, exhaustively -------------------------------------------------------
@pytest.mark.parametrize("fmt", FMTS)
def test_fast2sum_and_two_sum_every_pair(orc, fmt):
    f = F[fmt]
    fin = np.array(f.finite(), np.uint16)
    aa, bb = np.repeat(fin, fin.size), np.tile(fin, fin.size)
    va, vb = f64(orc, aa, fmt), f64(orc, bb, fmt)
    x2, y2 = orc.two_sum(aa, bb, fmt=fmt)
    vx, vy = f64(orc, x2, fmt), f64(orc, y2, fmt)
    ok = np.isfinite(vx) & np.isfinite(vy)                 # neither the sum nor an intermediate left the range
    assert ok.mean() > 0.9
    # TwoSum's one hazard: x is finite but x - a overflows (only next to the largest magnitude)
    assert np.count_nonzero(np.isfinite(vx) & ~np.isfinite(vy)) <= 4
    assert np.array_equal((vx + vy)[ok], (va + vb)[ok])    # exact: fp64 holds all these sums
    srt = np.abs(va) >= np.abs(vb)
    x1, y1 = orc.fast2sum(aa[srt], bb[srt], fmt=fmt)
    ok1 = np.isfinite(f64(orc, x1, fmt))
    with np.errstate(invalid="ignore"):
        assert np.array_equal((f64(orc, x1, fmt) + f64(orc, y1, fmt))[ok1], (va + vb)[srt][ok1])
    assert np.array_equal(x1, x2[srt])
    # non-overlap: |y| <= ulp(x)/2
    pick = rng.integers(0, x1.size, 500)
    for i in pick:
        if ok1[i] and f.value(int(x1[i])) != 0:
            assert abs(f.value(int(y1[i]))) <= f.ulp(f.value(int(x1[i]))) / 2


@pytest.mark.parametrize("fmt", FMTS)
def test_two_prod_fma_every_pair(orc, fmt):
    f = F[fmt]
    fin = np.array(f.finite(), np.uint16)
    aa, bb = np.repeat(fin, fin.size), np.tile(fin, fin.size)
    x, e = orc.two_prod_fma(aa, bb, fmt=fmt)
    assert np.array_equal(x, orc.binop(2, aa, bb, fmt=fmt))
    va, vb, vx, ve = (f64(orc, t, fmt) for t in (aa, bb, x, e))
    err = va * vb - vx                                   # exact in fp64
    ok = np.isfinite(vx)
    # e is the error rounded once; where the error is itself a number of the format, the pair is exact
    want_e = orc.R_array(err[ok].astype(np.float32), fmt=fmt)          # err has few bits: exact in fp32
    zero = err[ok] == 0
    assert np.array_equal(e[ok][~zero], want_e[~zero]) and np.all((e[ok][zero] & 0x7F) == 0)
    exact = f64(orc, want_e, fmt) == err[ok]
    assert exact.mean() > 0.5
    with np.errstate(invalid="ignore"):
        assert np.array_equal((vx + ve)[ok][exact], (va * vb)[ok][exact])


@pytest.mark.parametrize("fmt", FMTS)
def test_grow_keeps_what_one_component_loses(orc, fmt):
    f = F[fmt]
    one = f.nearest(1)
    small = f.nearest(Fraction(1, 64))                     # far below half an ulp of 1
    x, y = np.array([one], np.uint16), np.array([0], np.uint16)
    plain = np.array([one], np.uint16)
    a = np.array([small], np.uint16)
    for _ in range(8):
        x, y = orc.grow(x, y, a, fmt=fmt)
        plain = orc.binop(0, plain, a, fmt=fmt)
    assert plain[0] == one                                 # every addition was lost (Def. 3.2)
    assert f.value(int(x[0])) + f.value(int(y[0])) == 1 + Fraction(8, 64)
    # random valid triples (|a| <= |x|, (x, y) non-overlapping): the result is non-overlapping again
    fin = np.array(f.finite(), np.uint16)
    xs, ys, az = rng.choice(fin, 20000), rng.choice(fin, 20000), rng.choice(fin, 20000)
    vx, vy, va = f64(orc, xs, fmt), f64(orc, ys, fmt), f64(orc, az, fmt)
    gx, gy = orc.grow(xs, ys, az, fmt=fmt)
    checked = 0
    for i in range(xs.size):
        if checked == 500:
            break
        if vx[i] == 0 or abs(va[i]) > abs(vx[i]) or abs(f.value(int(ys[i]))) > f.ulp(f.value(int(xs[i]))) / 2:
            continue
        if f.is_nan(int(gx[i])) or f.is_inf(int(gx[i])) or f.is_nan(int(gy[i])) or f.value(int(gx[i])) == 0:
            continue
        assert abs(f.value(int(gy[i]))) <= f.ulp(f.value(int(gx[i]))) / 2, (hex(xs[i]), hex(ys[i]), hex(az[i]))
        checked += 1
    assert checked == 500
    assert vy.shape == vx.shape


# ---- scalars and the step ------------------------------------------------------------------------------
def test_scalar_patterns_by_hand(orc):
    s = orc.scalars(3e-4, 0.9, 0.95, 1e-8, 0.1, 1, fmt=E5M2)
    # E5M2 near 1 has steps of 1/8 below and 1/4 above: 0.95 -> 1.0; the rest, -0.05, lies in
    # [2^-5, 2^-4) with steps of 2^-7: 6.4 steps -> 6 steps = 0.046875 = 1.5 * 2^-5
    assert s["b2"] == 0x3C and s["b2l"] == 0x80 | (10 << 2) | 2
    assert s["e"] == 0                                         # 1e-8 is far below the least subnormal 2^-16
    assert s["b1"] == F[E5M2].nearest(Fraction(0.9)) == 0x3B   # 0.875
    assert s["na"] == 0x80 | F[E5M2].nearest(Fraction(3e-4))
    s = orc.scalars(3e-4, 0.9, 0.95, 1e-8, 0.1, 1, fmt=E4M3)
    # E4M3 in [0.5, 1) has steps of 1/16: 0.95 -> 15/16 = 1.875 * 2^-1; the rest 0.0125 is subnormal
    # (steps of 2^-9): 6.4 steps -> 6
    assert s["b2"] == (6 << 3) | 7 and s["b2l"] == 6
    assert s["na"] == 0x80                                     # 3e-4 is below half the least subnormal 2^-9: lr becomes -0
    assert s["lam"] == F[E4M3].nearest(Fraction(0.1))


@pytest.mark.parametrize("fmt", FMTS)
def test_one_step_by_hand_and_the_kept_update(orc, fmt):
    f = F[fmt]
    bits = lambda v: np.array([f.nearest(Fraction(v))], np.uint16)
    val = lambda h: f.value(int(h[0]))
    hyper = (0.5, 0.5, 0.5, 0.0, 0.0)
    theta, dth, m, v, g = bits(1), bits(0), bits(0), bits(0), bits(0.25)
    delta = np.zeros(1, np.uint16)
    orc.adamw_step(theta, dth, m, v, None, g, orc.LIGHT | orc.step_flag(fmt), hyper, 1, delta_out=delta)
    # m = 0.125, v = 0.03125, both bias corrections 0.5: m_hat = 0.25, v_hat = 0.0625, root 0.25, ratio 1, delta = -0.5
    assert val(m) == Fraction(1, 8) and val(v) == Fraction(1, 32) and val(delta) == Fraction(-1, 2)
    assert val(theta) == Fraction(1, 2) and val(dth) == 0
    hyper = (2.0 ** -6, 0.5, 0.5, 0.0, 0.0)                  # an update of 2^-6: below half an ulp of 1 in both formats
    theta, dth, m, v = bits(1), bits(0), bits(0), bits(0)
    orc.adamw_step(theta, dth, m, v, None, g, orc.LIGHT | orc.step_flag(fmt), hyper, 1)
    assert val(theta) == 1 and val(dth) == Fraction(-1, 64)
    plain, pm, pv = bits(1), bits(0), bits(0)
    orc.adamw_step(plain, None, pm, pv, None, g, orc.BF16 | orc.step_flag(fmt), hyper, 1)
    assert val(plain) == 1                                    # lost arithmetic
    acc = orc.EdqAccumulator(fmt=fmt)
    acc.add(bits(-1 / 64), bits(1), bits(0), theta, dth)
    assert acc.lost.value == 0 and abs(acc.value() - 1 / 64) < 1e-15
    acc = orc.EdqAccumulator(fmt=fmt)
    acc.add(bits(-1 / 64), bits(1), None, plain, None)
    assert acc.lost.value == 1 and acc.value() == 0.0


@pytest.mark.parametrize("fmt", FMTS)
def test_e4m3_overflow_is_nan_and_e5m2_overflow_is_infinity(orc, fmt):
    f = F[fmt]
    big = np.array([f.max_bits], np.uint16)
    s = orc.binop(0, big, big, fmt=fmt)
    p = orc.binop(2, big, big, fmt=fmt)
    if fmt == E5M2:
        assert s[0] == 0x7C and p[0] == 0x7C
        assert orc.binop(1, s, s, fmt=fmt)[0] == 0x7E         # inf - inf
    else:
        assert s[0] == 0x7F and p[0] == 0x7F
        assert np.isnan(orc.widen(0x7F, fmt=fmt)) and np.isnan(orc.widen(0xFF, fmt=fmt))


def _same_patterns(orc, fmt, got, want):
    """Equal 8-bit patterns, any NaN matching any NaN."""
    nan_got, nan_want = np.isnan(orc.widen_array(got, fmt=fmt)), np.isnan(orc.widen_array(want, fmt=fmt))
    return (got == want) | (nan_got & nan_want)


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("ulps", [0, 1, -1, 2, -2])
def test_quotient_through_an_fp32_reciprocal_and_an_fp16_rounding(orc, fmt, ulps):
    """What the GPU kernels rely on for F(a / b): fl32(a * r), rounded to fp16 and then to the format, is
    F(a / b) for every one of the 256 x 256 (a, b) as long as r is within two units in the last place of
    1/b -- the exact ties among the quotients are fp16 numbers, so the fp16 rounding restores them and
    the last rounding sees them as ties; b = 0, infinite or NaN included.  IEEE fp32 and fp16 arithmetic
    only, so this holds on any machine (the hardware's reciprocal instruction is within one unit)."""
    v = orc.widen_array(ALL, fmt=fmt)
    a, b = np.repeat(v, 256), np.tile(v, 256)
    with np.errstate(all="ignore"):
        r = (1.0 / b.astype(np.float64)).astype(np.float32)
        moved = r.copy()
        for _ in range(abs(ulps)):
            moved = np.nextafter(moved, np.float32(np.inf if ulps > 0 else -np.inf) * np.sign(r).astype(np.float32))
        r = np.where(np.isfinite(r) & (r != 0), moved, r)
        q16 = (a * r).astype(np.float32).astype(np.float16)
    got = orc.R_array(q16.astype(np.float32), fmt=fmt)
    want = orc.binop(3, np.repeat(ALL, 256), np.tile(ALL, 256), fmt=fmt)
    assert _same_patterns(orc, fmt, got, want).all()


@pytest.mark.parametrize("fmt", FMTS)
def test_division_by_a_scalar_through_its_fp16_reciprocal(orc, fmt):
    """What the GPU kernels rely on for the two bias corrections: with r = RN16(1/b), one fp16
    multiplication a * r followed by the rounding to the format is F(a / b) for every a and every b whose
    reciprocal is an fp16 number -- all of E4M3, and all of E5M2 but +-2^-16 (the library sends a step
    with such a bias correction down its element path, which divides properly)."""
    v = orc.widen_array(ALL, fmt=fmt)
    a, b = np.repeat(v, 256), np.tile(v, 256)
    with np.errstate(all="ignore"):
        r16 = (1.0 / b.astype(np.float64)).astype(np.float16)
        prod = (a.astype(np.float64) * r16.astype(np.float64)).astype(np.float16)       # exact product, one rounding
    got = orc.R_array(prod.astype(np.float32), fmt=fmt)
    want = orc.binop(3, np.repeat(ALL, 256), np.tile(ALL, 256), fmt=fmt)
    bad_b = np.unique(np.abs(b[~_same_patterns(orc, fmt, got, want)]))
    assert list(bad_b) == ([] if fmt == orc.FMT_E4M3 else [2.0 ** -16])
