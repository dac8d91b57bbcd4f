"""Pins for the oracle's rounding primitives R, B and the single bf16 operation F(a o b).

Independent references used here: exact rational arithmetic with a nearest-
neighbour search over the table of all bf16 values (helpers.nearest_bf16),
torch's own fp32->bf16 cast, the values printed in the paper
(tests/golden/paper_values.txt), and fp64 arithmetic followed by one rounding
(valid because a correctly rounded p-bit result of + - * / sqrt of 8-bit
operands re-rounds innocuously to 8 bits whenever p >= 2*8+2).
"""
import os
import random
from fractions import Fraction

import numpy as np
import pytest
import torch

import helpers as H

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def _f32_from_bits(b):
    return np.array([b], dtype=np.uint32).view(np.float32)[0]


# ---------------------------------------------------------------- helpers self-check
def test_reference_search_on_hand_cases():
    # 1 + 2^-8 is the midpoint of 1 and 1+2^-7: ties to even -> 1.0 (0x3F80)
    assert H.nearest_bf16(Fraction(1) + Fraction(1, 256)) == 0x3F80
    # 1 + 3*2^-8 is the midpoint of 1+2^-7 (odd) and 1+2^-6 (even) -> 0x3F82
    assert H.nearest_bf16(Fraction(1) + Fraction(3, 256)) == 0x3F82
    assert H.nearest_bf16(Fraction(1) + Fraction(1, 256) + Fraction(1, 2 ** 40)) == 0x3F81
    assert H.nearest_bf16(Fraction(0)) == 0
    assert H.nearest_bf16(Fraction(-3)) == 0xC040
    # least subnormal 2^-133 and half of it (tie to even -> 0)
    assert H.nearest_bf16(Fraction(1, 2 ** 133)) == 0x0001
    assert H.nearest_bf16(Fraction(1, 2 ** 134)) == 0x0000
    assert H.nearest_bf16(Fraction(3, 2 ** 134)) == 0x0002
    # overflow threshold
    big = H.bf16_bits_to_fraction(0x7F7F)
    assert H.nearest_bf16(big + Fraction(2) ** 118) == 0x7F7F      # below the midpoint (2^119)
    assert H.nearest_bf16(big + Fraction(2) ** 119) == 0x7F80


def test_numpy_rounding_matches_rational_search():
    rng = random.Random(1)
    xs = []
    for _ in range(3000):
        e = rng.randint(-140, 130)
        xs.append(rng.choice((-1, 1)) * rng.random() * 2.0 ** e if e > -1000 else 0.0)
    # exact ties and near ties
    for h in (0x3F80, 0x3F81, 0x0001, 0x007F, 0x0080, 0x7F7E, 0x7F7F, 0x1234):
        a, b = H.bf16_bits_to_fraction(h), H.bf16_bits_to_fraction(min(h + 1, 0x7F7F))
        mid = float((a + b) / 2)
        xs += [mid, np.nextafter(mid, np.inf), np.nextafter(mid, -np.inf), -mid]
    xs = np.array(xs, dtype=np.float64)
    got = H.np_round_f64_to_bf16(xs)
    for x, g in zip(xs.tolist(), got.tolist()):
        assert g == H.nearest_bf16(Fraction(x)), (x, hex(g))


# ---------------------------------------------------------------- paper's printed values
def test_paper_printed_values(orc):
    rows = H.read_golden(GOLD)
    seen = set()
    for kind, inputs, expected, _where in rows:
        seen.add(kind)
        if kind == "round":
            got = orc.widen(orc.B(float(inputs)))
            digits = len(expected.split(".")[1])
            assert round(got, digits) == float(expected), (inputs, got)
        elif kind == "add":
            a, b = (float(t) for t in inputs.split())
            r = orc.binop(orc.ADD, np.array([orc.B(a)], np.uint16), np.array([orc.B(b)], np.uint16))
            assert orc.widen(r[0]) == float(expected)
        elif kind == "ulp":
            x = float(inputs)
            want = 2.0 ** int(expected.split("^")[1]) if "^" in expected else float(expected)
            h = orc.B(x)
            assert orc.widen(h) == x
            assert orc.widen(h + 1) - orc.widen(h) == want        # spacing to the next bf16
            assert float(H.ulp_bf16(Fraction(x))) == want
        elif kind == "expand":
            x = float(inputs)
            hi_s, lo_s = expected.split()
            hi = orc.widen(orc.B(x))
            lo = orc.widen(orc.B(x - hi))
            nd = lambda s: len(s.split(".")[1]) if "." in s else 0
            assert round(hi, nd(hi_s)) == float(hi_s), (x, hi)
            assert round(lo, nd(lo_s)) == float(lo_s), (x, lo)
            s = orc.scalars(1e-3, 0.9, x, 1e-8, 0.0, 1)
            assert orc.widen(s["b2"]) == hi and orc.widen(s["b2l"]) == lo
        elif kind == "lostmul":
            al = float(inputs)
            one = np.array([orc.B(1.0)], np.uint16)
            if expected == "lost":
                f = np.array([orc.B(1.0 - al)], np.uint16)
                assert orc.binop(orc.MUL, one, f)[0] == one[0]
                # and as a subtraction theta - alpha*lambda*theta
                d = np.array([orc.B(al)], np.uint16)
                assert orc.binop(orc.SUB, one, d)[0] == one[0]
            else:
                # half an ulp of 1.0 is the least decrement that can survive; anything smaller is lost
                assert round(2.0 ** -8, 4) == al
                d_ok = np.array([orc.B(2.0 ** -8 * 1.01)], np.uint16)
                d_lost = np.array([orc.B(2.0 ** -10)], np.uint16)
                assert orc.binop(orc.SUB, one, d_ok)[0] != one[0]
                assert orc.binop(orc.SUB, one, d_lost)[0] == one[0]
    assert {"round", "add", "ulp", "expand", "lostmul"} <= seen


# ---------------------------------------------------------------- R : fp32 -> bf16
def test_R_against_torch_cast(orc):
    """All 2^16 upper halves x 64 lower halves (edge values + random) = 4M fp32 patterns."""
    rng = np.random.default_rng(0)
    lows = np.unique(np.concatenate([np.array([0, 1, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x4000, 0xC000]),
                                     rng.integers(0, 1 << 16, 56)])).astype(np.uint32)
    highs = np.arange(1 << 16, dtype=np.uint32) << 16
    bits = (highs[:, None] | lows[None, :]).reshape(-1)
    f = bits.view(np.float32)
    ref = H.torch_to_u16(torch.from_numpy(f.copy()).to(torch.bfloat16))
    got = orc.R_array(f)
    nan = np.isnan(f)
    assert np.array_equal(got[~nan], ref[~nan])
    assert nan.sum() > 0 and np.all(got[nan] == 0x7FC0)


def test_R_against_rational_search(orc):
    rng = random.Random(2)
    cases = [0x00000000, 0x80000000, 0x00000001, 0x00007FFF, 0x00008000, 0x00008001, 0x00018000,
             0x007F8000, 0x007FFFFF, 0x00800000, 0x3F808000, 0x3F818000, 0x3F80FFFF, 0x7F7F7FFF,
             0x7F7F8000, 0x7F7FFFFF, 0x7F800000, 0xFF800000]
    cases += [rng.getrandbits(32) for _ in range(4000)]
    for b in cases:
        f = _f32_from_bits(b)
        if np.isnan(f):
            assert orc.R(f) == 0x7FC0
            continue
        if np.isinf(f):
            assert orc.R(f) == (0x7F80 | (0x8000 if f < 0 else 0))
            continue
        want = H.nearest_bf16(Fraction(float(f)))
        if float(f) == 0.0 and (b >> 31):
            want |= 0x8000
        assert orc.R(f) == want, hex(b)


def test_R_is_identity_on_bf16_and_monotone(orc):
    hs = np.arange(0, 0x7F81, dtype=np.uint16)
    vals = H.u16_to_f32(hs)
    for h, v in zip(hs[::37].tolist(), vals[::37].tolist()):
        assert orc.R(v) == h
    rng = np.random.default_rng(3)
    f = np.sort(rng.standard_normal(2000).astype(np.float32) * np.float32(1e3))
    r = [orc.widen(orc.R(x)) for x in f.tolist()]
    assert all(r[i] <= r[i + 1] for i in range(len(r) - 1))


# ---------------------------------------------------------------- B : fp64 -> bf16, one rounding
def test_B_against_rational_search(orc):
    rng = random.Random(4)
    xs = [0.0, -0.0, 1.0, -1.0, 0.999, 0.99, 0.95, 0.1, 1e-8, 3e-4, 2.0 ** -133, 2.0 ** -134, 3 * 2.0 ** -134,
          2.0 ** -126, 2.0 ** -126 * (1 - 2.0 ** -9), 3.3e38, 3.4e38, 1e39, 1e-45, 1e-300, 1e300]
    for _ in range(4000):
        xs.append(rng.choice((-1, 1)) * rng.random() * 2.0 ** rng.randint(-140, 129))
    for x in xs:
        want = H.nearest_bf16(Fraction(x))
        if x == 0.0 and np.signbit(x):
            want |= 0x8000
        assert orc.B(x) == want, x
    assert orc.B(float("inf")) == 0x7F80 and orc.B(float("-inf")) == 0xFF80
    assert orc.B(float("nan")) == 0x7FC0


def test_B_does_not_double_round(orc):
    # x just above the midpoint between 1.0 and 1+2^-7: a cast through fp32 first would land on the
    # midpoint (tie -> 1.0); a single rounding must give 1+2^-7.
    x = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert float(np.float32(x)) == 1.0 + 2.0 ** -8
    assert orc.B(x) == 0x3F81
    x = 1.0 + 3 * 2.0 ** -8 - 2.0 ** -40      # just below a midpoint whose tie would go up
    assert orc.B(x) == 0x3F81


# ---------------------------------------------------------------- F(a o b)
def _interesting_pairs(n, seed):
    rng = np.random.default_rng(seed)
    finite = H.all_finite_bf16()
    a = rng.choice(finite, n)
    b = rng.choice(finite, n)
    # half of the pairs get exponents close to each other so that the operations really round
    k = n // 2
    ea = rng.integers(1, 254, k)
    eb = np.clip(ea + rng.integers(-10, 11, k), 1, 254)
    a[:k] = (ea << 7 | rng.integers(0, 128, k) | (rng.integers(0, 2, k) << 15)).astype(np.uint16)
    b[:k] = (eb << 7 | rng.integers(0, 128, k) | (rng.integers(0, 2, k) << 15)).astype(np.uint16)
    # subnormals and zeros
    a[k:k + 50] = rng.integers(0, 0x100, 50).astype(np.uint16)
    b[k + 25:k + 75] = rng.integers(0, 0x100, 50).astype(np.uint16)
    return a.astype(np.uint16), b.astype(np.uint16)


@pytest.mark.parametrize("opname", ["add", "sub", "mul", "div"])
def test_F_binary_against_exact_rationals(orc, opname):
    op = {"add": orc.ADD, "sub": orc.SUB, "mul": orc.MUL, "div": orc.DIV}[opname]
    a, b = _interesting_pairs(6000, 10 + op)
    got = orc.binop(op, a, b)
    checked = 0
    for x, y, g in zip(a.tolist(), b.tolist(), got.tolist()):
        fx, fy = H.bf16_bits_to_fraction(x), H.bf16_bits_to_fraction(y)
        if opname == "div" and fy == 0:
            continue
        exact = {"add": fx + fy, "sub": fx - fy, "mul": fx * fy, "div": fx / fy if fy else None}[opname]
        if exact == 0:
            assert g & 0x7FFF == 0          # sign of zero is checked by the IEEE-special test
            continue
        assert g == H.nearest_bf16(exact), (opname, hex(x), hex(y), hex(g))
        checked += 1
    assert checked > 5000


def test_F_sqrt_against_exact_rationals(orc):
    pos = np.arange(1, 0x7F80, dtype=np.uint16)          # every positive finite bf16
    got = orc.binop(orc.SQRT, pos)
    for x, g in zip(pos[::5].tolist(), got[::5].tolist()):
        fx = H.bf16_bits_to_fraction(x)
        c = H.bf16_bits_to_fraction(g)
        # c is the nearest bf16 to sqrt(fx)  <=>  fx lies between the squares of c's two rounding midpoints
        lo = (c + H.bf16_bits_to_fraction(g - 1)) / 2
        hi = (c + H.bf16_bits_to_fraction(g + 1)) / 2
        assert lo * lo <= fx <= hi * hi, hex(x)
        assert not (lo * lo == fx or hi * hi == fx)       # a square root of a bf16 is never a midpoint


def test_F_ieee_specials(orc):
    u = lambda *v: np.array(v, dtype=np.uint16)
    pz, nz, inf, ninf, one, nan = 0x0000, 0x8000, 0x7F80, 0xFF80, 0x3F80, 0x7FC0
    assert orc.binop(orc.ADD, u(pz), u(nz))[0] == pz
    assert orc.binop(orc.ADD, u(nz), u(nz))[0] == nz
    assert orc.binop(orc.SUB, u(one), u(one))[0] == pz
    assert orc.binop(orc.MUL, u(nz), u(one))[0] == nz
    assert orc.binop(orc.DIV, u(one), u(pz))[0] == inf
    assert orc.binop(orc.DIV, u(one), u(nz))[0] == ninf
    assert orc.binop(orc.DIV, u(pz), u(pz))[0] == nan
    assert orc.binop(orc.SUB, u(inf), u(inf))[0] == nan
    assert orc.binop(orc.MUL, u(inf), u(pz))[0] == nan
    assert orc.binop(orc.SQRT, u(nz))[0] == nz
    assert orc.binop(orc.SQRT, u(0xBF80))[0] == nan
    assert orc.binop(orc.SQRT, u(inf))[0] == inf
    assert orc.binop(orc.ADD, u(0x7F7F), u(0x7F7F))[0] == inf          # overflow
    assert orc.binop(orc.ADD, u(0xFFFF), u(one))[0] == nan            # any NaN in -> canonical NaN out


@pytest.mark.parametrize("opname", ["add", "mul", "div"])
def test_F_sweep_against_fp64_route(orc, opname):
    """Rows of the full 2^16 x 2^16 table: fp32-then-R must equal fp64-then-one-rounding.
    MCF_FULL_SWEEP=1 runs every row (minutes); the default takes 256 seeded rows plus edge rows."""
    op = {"add": orc.ADD, "mul": orc.MUL, "div": orc.DIV}[opname]
    finite = H.all_finite_bf16()
    fvals = H.u16_to_f64(finite)
    if os.environ.get("MCF_FULL_SWEEP") == "1":
        rows = finite
    else:
        rng = np.random.default_rng(20)
        rows = np.unique(np.concatenate([rng.choice(finite, 256),
                                         np.array([0, 1, 0x7F, 0x80, 0x3F80, 0x3F81, 0x7F7F, 0x8001, 0xBF80],
                                                  dtype=np.uint16)]))
    for a in rows.tolist():
        av = H.u16_to_f64(np.array([a], np.uint16))[0]
        aa = np.full(finite.shape, a, dtype=np.uint16)
        got = orc.binop(op, aa, finite)
        with np.errstate(all="ignore"):
            ref64 = {"add": av + fvals, "mul": av * fvals, "div": av / fvals}[opname]
        ok = ~np.isnan(ref64)
        want = H.np_round_f64_to_bf16(ref64[ok])
        nz = ref64[ok] != 0                          # signed-zero results are pinned in test_F_ieee_specials
        assert np.array_equal(got[ok][nz], want[nz]), hex(a)
        assert np.all((got[ok][~nz] & 0x7FFF) == 0)
        assert np.all(got[~ok] == 0x7FC0)


def test_fp_environment_and_threads(orc):
    assert orc.fp_env_ok()
    # subnormal operands and results survive an operation
    tiny = np.array([0x0001], np.uint16)                  # 2^-133
    two = np.array([0x4000], np.uint16)
    assert orc.binop(orc.MUL, tiny, two)[0] == 0x0002
    assert orc.binop(orc.ADD, tiny, tiny)[0] == 0x0002


# ------------------------------------------------------------------ quotients below the normal range
def _bf16_as_f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


@pytest.mark.parametrize("ulps", [0, 1, -1])
def test_small_quotients_through_a_reciprocal(orc, ulps):
    """What the GPU's restricted arithmetic mode relies on below the normal range: for every bf16 a and every
    bf16 b with 2^-126 <= |b| <= 2^126 whose quotient lies below 2^-125 (subnormal results, and those that
    round to zero or up to the least normal number), R(fl32(a * r)) = F(a / b) for r anywhere within one unit
    in the last place of 1/b -- except that a power of two must have its exact reciprocal, which is the
    only case where a quotient this size can sit on a rounding tie that the product's own rounding does
    not restore.  IEEE fp32 multiplication with subnormal results only, so this holds on any machine."""
    bad = checked = 0
    with np.errstate(all="ignore"):
        for eb in range(1, 254):                                   # biased exponent of b
            mant = np.arange(128) if eb < 253 else np.arange(1)    # 2^126 itself is the last divisor allowed
            b_bits = ((eb << 7) | mant).astype(np.uint16)
            lo_e, hi_e = max(0, eb - 136), min(254, eb - 124)      # |a/b| within [2^-137, 2^-123)
            if hi_e < lo_e:
                continue
            a_bits = np.array([(e << 7) | m for e in range(lo_e, hi_e + 1) for m in range(128)], np.uint16)
            a_bits = a_bits[a_bits != 0]
            a_bits = np.concatenate([a_bits, a_bits | 0x8000])
            A, B = [x.ravel() for x in np.meshgrid(a_bits, b_bits, indexing="ij")]
            fa, fb = _bf16_as_f32(A), _bf16_as_f32(B)
            r = (1.0 / fb.astype(np.float64)).astype(np.float32)
            if ulps:
                moved = np.nextafter(r, np.float32(np.inf if ulps > 0 else -np.inf))
                r = np.where((B & 0x7F) == 0, r, moved)
            got = orc.R_array((fa * r).astype(np.float32))
            want = orc.binop(orc.DIV, A, B)
            bad += int(np.sum(got != want))
            checked += A.size
    assert checked > 5e7 and bad == 0


def test_small_quotients_by_a_bias_correction(orc):
    """The same for the two divisions by a bias correction bc in [2^-60, 1], whose reciprocal the host
    rounds correctly: R(fl32(a * fl32(1/bc))) = F(a / bc) for every bf16 a small enough for the quotient to
    be subnormal (|a| < 2^-125)."""
    a_bits = np.arange(1, 3 << 7, dtype=np.uint16)                 # biased exponents 0..2: up to 2^-124
    a_bits = np.concatenate([a_bits, a_bits | 0x8000])
    bc_bits = np.arange((127 - 60) << 7, (127 << 7) + 1, dtype=np.uint16)
    A, B = [x.ravel() for x in np.meshgrid(a_bits, bc_bits, indexing="ij")]
    with np.errstate(all="ignore"):
        r = (1.0 / _bf16_as_f32(B).astype(np.float64)).astype(np.float32)
        got = orc.R_array((_bf16_as_f32(A) * r).astype(np.float32))
    assert np.array_equal(got, orc.binop(orc.DIV, A, B))


def test_every_quotient_by_a_bias_correction_through_its_reciprocal(orc):
    """Lines 10-11 of Alg. 2 in the GPU's restricted arithmetic mode, exhaustively: for EVERY bf16 pattern a
    (zeros, subnormals, infinities and NaN included) and every bf16 bias correction bc in [2^-60, 1] -- the
    range in which the host lets that mode run -- the product of a with the correctly rounded fp32
    reciprocal of bc, rounded to bf16, is F(a / bc).  5.0e8 pairs of pure IEEE fp32 arithmetic; a NaN on one
    side must be a NaN on the other (the kernel then redoes the slot and stores the one NaN pattern)."""
    a_bits = np.arange(1 << 16, dtype=np.uint16)
    fa = _bf16_as_f32(a_bits)
    bc_all = np.arange((127 - 60) << 7, (127 << 7) + 1, dtype=np.uint16)
    assert bc_all.size == 60 * 128 + 1
    bad = checked = 0
    with np.errstate(all="ignore"):
        for i in range(0, bc_all.size, 64):
            bc = bc_all[i:i + 64]
            r = (1.0 / _bf16_as_f32(bc).astype(np.float64)).astype(np.float32)           # what the host passes
            got = orc.R_array((fa[None, :] * r[:, None]).astype(np.float32).ravel())
            want = orc.binop(orc.DIV, np.tile(a_bits, bc.size), np.repeat(bc, a_bits.size))
            bad += int(np.count_nonzero(got != want))
            checked += got.size
    assert checked == (60 * 128 + 1) * 65536 and bad == 0
