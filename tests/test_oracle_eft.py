"""Pins for the oracle's error-free transformations: Fast2Sum (Thm 4.1), TwoSum (Alg. 3),
Grow (Alg. 1), TwoProdFMA (Alg. 6) and Mul (Alg. 8).

References: exact sums and products in float64 (exact for bf16 operands whose exponents lie
within ~40 binades of each other, which the windows below guarantee), the paper's worked
expansion of 0.999, and a brute-force fp64 accumulation.
"""
import numpy as np

import helpers as H


def _ulp_arr(x):
    """bf16 spacing at |x| (float64 array), Def. 3.1 with 7 stored bits."""
    a = np.abs(x)
    _, e = np.frexp(a)
    e = e.astype(np.int64) - 1
    return np.where(a == 0, 2.0 ** -133, np.ldexp(1.0, (np.maximum(e, -126) - 7).astype(np.int32)))


def _grid(vals):
    a = np.repeat(vals, vals.size)
    b = np.tile(vals, vals.size)
    return a, b


def test_fast2sum_exhaustive_window(orc):
    """Every ordered pair of bf16 values with exponents in [-6, 6], both signs, plus zero: 11M pairs."""
    vals = np.concatenate([H.bf16_window(-6, 6), np.array([0, 0x8000], np.uint16)])
    a, b = _grid(vals)
    x, y = orc.fast2sum(a, b)
    fa, fb, fx, fy = (H.u16_to_f64(t) for t in (a, b, x, y))
    # x is the correctly rounded sum for every pair
    assert np.array_equal(x[(fa + fb) != 0], H.np_round_f64_to_bf16((fa + fb)[(fa + fb) != 0]))
    ordered = np.abs(fa) >= np.abs(fb)
    assert ordered.sum() > 5_000_000
    # Thm 4.1: exact, and the error term is at most half an ulp of the sum
    assert np.array_equal((fx + fy)[ordered], (fa + fb)[ordered])
    assert np.all(np.abs(fy[ordered]) <= _ulp_arr(fx[ordered]) / 2)
    # the precondition matters: with the operands swapped exactness does fail somewhere
    assert np.any((fx + fy)[~ordered] != (fa + fb)[~ordered])


def test_fast2sum_wide_gaps_and_subnormals(orc):
    rng = np.random.default_rng(5)
    big = H.bf16_window(-20, 20)
    a = rng.choice(big, 400_000)
    b = rng.choice(big, 400_000)
    sub = np.concatenate([np.arange(0, 0x180, dtype=np.uint16), np.arange(0x8000, 0x8180, dtype=np.uint16)])
    sa, sb = _grid(sub)
    a = np.concatenate([a, sa])
    b = np.concatenate([b, sb])
    fa, fb = H.u16_to_f64(a), H.u16_to_f64(b)
    swap = np.abs(fa) < np.abs(fb)
    a2 = np.where(swap, b, a)
    b2 = np.where(swap, a, b)
    x, y = orc.fast2sum(a2, b2)
    fx, fy = H.u16_to_f64(x), H.u16_to_f64(y)
    assert np.array_equal(fx + fy, fa + fb)
    assert np.all(np.abs(fy) <= _ulp_arr(fx) / 2)


def test_fast2sum_worked_expansion_of_0p999(orc):
    """Sec. 2.2 / Table 2: 0.999 = (1.0, -0.001) as a two-component bf16 number."""
    one = np.array([orc.B(1.0)], np.uint16)
    lo = np.array([orc.B(0.999 - 1.0)], np.uint16)
    x, y = orc.fast2sum(one, lo)
    assert orc.widen(x[0]) == 1.0
    assert round(orc.widen(y[0]), 3) == -0.001
    assert abs((orc.widen(x[0]) + orc.widen(y[0])) - 0.999) < 2.0 ** -17


def test_two_sum_matches_fast2sum_and_needs_no_order(orc):
    vals = np.concatenate([H.bf16_window(-5, 5), np.array([0], np.uint16)])
    a, b = _grid(vals)
    x, y = orc.two_sum(a, b)
    fa, fb, fx, fy = (H.u16_to_f64(t) for t in (a, b, x, y))
    assert np.array_equal(fx + fy, fa + fb)                  # exact for either order
    ordered = np.abs(fa) >= np.abs(fb)
    xf, yf = orc.fast2sum(a, b)
    nz = H.u16_to_f64(yf) != 0
    # identical expansion where Fast2Sum's precondition holds (sign of a zero error term aside)
    assert np.array_equal(x[ordered], xf[ordered])
    assert np.array_equal(y[ordered & nz], yf[ordered & nz])
    assert np.all(fy[ordered & ~nz] == 0)


def test_two_prod_fma_is_exact(orc):
    vals = H.bf16_window(-8, 8)
    rng = np.random.default_rng(6)
    a = rng.choice(vals, 2_000_000)
    b = rng.choice(vals, 2_000_000)
    x, e = orc.two_prod_fma(a, b)
    fa, fb, fx, fe = (H.u16_to_f64(t) for t in (a, b, x, e))
    assert np.array_equal(fx + fe, fa * fb)
    assert np.array_equal(x, H.np_round_f64_to_bf16(fa * fb))
    assert np.all(np.abs(fe) <= _ulp_arr(fx) / 2)


def test_mul_expansion(orc):
    rng = np.random.default_rng(7)
    n = 500_000
    hi = H.bf16_window(-10, 2)
    b1 = rng.choice(hi, n)
    # second components below half an ulp of the first
    f1 = H.u16_to_f64(b1)
    b2 = H.np_round_f64_to_bf16(_ulp_arr(f1) * rng.uniform(-0.5, 0.5, n) * 0.99)
    for beta2 in (0.999, 0.99, 0.95, 0.98):
        a1 = np.full(n, orc.B(beta2), np.uint16)
        a2 = np.full(n, orc.B(beta2 - orc.widen(orc.B(beta2))), np.uint16)
        x, e = orc.mul_expansion(a1, a2, b1, b2)
        fx, fe = H.u16_to_f64(x), H.u16_to_f64(e)
        exact = (H.u16_to_f64(a1) + H.u16_to_f64(a2)) * (f1 + H.u16_to_f64(b2))
        rel = np.abs((fx + fe) - exact) / np.abs(exact)
        assert rel.max() < 2.0 ** -13, rel.max()
        assert np.all(np.abs(fe) <= _ulp_arr(fx) / 2)       # result is a non-overlapping expansion
        # and much better than the one-component product
        plain = H.u16_to_f64(orc.binop(orc.MUL, a1, b1))
        assert np.median(np.abs(plain - exact) / np.abs(exact)) > 20 * np.median(rel)
    # collapse: zero second components reduce Mul to TwoProdFMA + Fast2Sum, which is exact
    z = np.zeros(n, np.uint16)
    a1 = np.full(n, orc.B(0.95), np.uint16)
    x, e = orc.mul_expansion(a1, z, b1, z)
    assert np.array_equal(H.u16_to_f64(x) + H.u16_to_f64(e), H.u16_to_f64(a1) * f1)


def test_mul_operand_roles(orc):
    """(a1,a2) x (b1,b2): the cross terms are a1*b2 and a2*b1 (Alg. 8 line 3), checked on values where
    swapping the roles of the second components would give a different answer."""
    u = lambda v: np.array([orc.B(v)], np.uint16)
    a1, a2, b1, b2 = u(1.0), u(-0.001), u(3.0), u(0.0078125)
    x, e = orc.mul_expansion(a1, a2, b1, b2)
    exact = (1.0 + orc.widen(a2[0])) * (3.0 + 0.0078125)
    assert abs(orc.widen(x[0]) + orc.widen(e[0]) - exact) < 2.0 ** -14 * exact
    wrong = 1.0 * 3.0 + 1.0 * orc.widen(a2[0]) + 3.0 * 0.0078125 * 0    # dropping a cross term is visible
    assert abs(wrong - exact) > 2.0 ** -9


def test_grow_identity_and_non_overlap(orc):
    """One Grow loses exactly the rounding error of its single inexact addition (y + v):
    (x'+y') - (x+y+a) = -(err of F(y (+) v)), and the result is non-overlapping (Def. 2.1)."""
    rng = np.random.default_rng(8)
    n = 2_000_000
    x = rng.choice(H.bf16_window(-8, 4), n)
    fx = H.u16_to_f64(x)
    y = H.np_round_f64_to_bf16(_ulp_arr(fx) * rng.uniform(-0.5, 0.5, n) * 0.99)
    # addends from the same size as x down to 2^-24 of it
    scale = 2.0 ** rng.uniform(-24, 0, n)
    a = H.np_round_f64_to_bf16(fx * scale * rng.choice([-1.0, 1.0], n) * 0.999)
    fa, fy = H.u16_to_f64(a), H.u16_to_f64(y)
    assert np.all(np.abs(fx) >= np.abs(fa))
    x2, y2 = orc.grow(x, y, a)
    f2x, f2y = H.u16_to_f64(x2), H.u16_to_f64(y2)
    # recompute the one inexact step independently in fp64: u = RN(x+a), v = x+a-u (exact), t = RN(y+v)
    u = H.u16_to_f64(H.np_round_f64_to_bf16(fx + fa))
    v = (fx + fa) - u
    t_exact = fy + v
    t = H.u16_to_f64(H.np_round_f64_to_bf16(np.where(t_exact == 0, 0.0, t_exact)))
    assert np.array_equal((f2x + f2y) - (fx + fy + fa), t - t_exact)
    assert np.all(np.abs((f2x + f2y) - (fx + fy + fa)) <= _ulp_arr(t) / 2)
    assert np.all(np.abs(f2y) <= _ulp_arr(f2x) / 2)


def test_mcf_accumulation_against_fp64_sum(orc):
    """Sec. 3 / Sec. 4: adding many small updates to a large weight.  Plain bf16 addition loses every
    one of them (lost arithmetic, Def. 3.2); Grow loses at most half an ulp of the SECOND component per
    step (about 2^-17 of the sum), which over thousands of steps is a random walk far below one bf16 ulp."""
    rng = np.random.default_rng(9)
    n_acc, steps = 512, 4_000
    x = np.full(n_acc, orc.B(200.0), np.uint16)
    y = np.zeros(n_acc, np.uint16)
    plain = x.copy()
    exact = np.full(n_acc, 200.0)
    for _ in range(steps):
        a = H.np_round_f64_to_bf16(rng.uniform(0.05, 0.15, n_acc))         # each below ulp(200)/2 = 0.5
        exact += H.u16_to_f64(a)
        x, y = orc.grow(x, y, a)
        plain = orc.binop(orc.ADD, plain, a)
    assert np.all(H.u16_to_f64(plain) == 200.0)                            # F(200 (+) 0.1) = 200, every time
    got = H.u16_to_f64(x) + H.u16_to_f64(y)
    assert exact.min() > 550.0
    rel = np.abs(got - exact) / exact
    # worst case: every step loses a full half-ulp of y (|y| <= 2 here, so <= 2^-8 each) in the same direction
    assert np.all(np.abs(got - exact) <= steps * 2.0 ** -8)
    assert rel.max() < 2.0 ** -10 and np.median(rel) < 2.0 ** -12, (rel.max(), np.median(rel))
    assert np.all(np.abs(H.u16_to_f64(y)) <= _ulp_arr(H.u16_to_f64(x)) / 2)


def test_scaling_is_mul_by_a_one_component_number(orc):
    """Alg. 7 is Alg. 8 with b = (v, 0): the same bits wherever no signed zero is involved, and accurate to the
    resolution of a two-component number."""
    rng = np.random.default_rng(12)
    n = 400_000
    a1 = rng.choice(H.bf16_window(-6, 6), n)
    f1 = H.u16_to_f64(a1)
    a2 = H.np_round_f64_to_bf16(_ulp_arr(f1) * rng.uniform(-0.5, 0.5, n) * 0.99)
    v = rng.choice(H.bf16_window(-6, 6), n)
    x, e = orc.scaling(v, a1, a2)
    xm, em = orc.mul_expansion(a1, a2, v, np.zeros(n, np.uint16))
    nz = (H.u16_to_f64(e) != 0) & (H.u16_to_f64(a2) != 0)
    assert np.array_equal(x, xm) and np.array_equal(e[nz], em[nz])
    exact = (f1 + H.u16_to_f64(a2)) * H.u16_to_f64(v)
    rel = np.abs(H.u16_to_f64(x) + H.u16_to_f64(e) - exact) / np.abs(exact)
    assert rel.max() < 2.0 ** -14
    assert np.all(np.abs(H.u16_to_f64(e)) <= _ulp_arr(H.u16_to_f64(x)) / 2)
