"""Pins for the oracle's effective descent quality (Def. 3.3, Eq. 2-3)."""
import math
from fractions import Fraction

import numpy as np

import helpers as H


def _bits(orc, vals):
    return np.array([orc.B(v) for v in vals], np.uint16)


def test_edq_equals_update_norm_without_imprecision(orc):
    """Sec. 3.2: with no lost arithmetic the effective update is the intended one and EDQ = ||delta||."""
    theta = _bits(orc, [1.0, -2.0, 0.5, 4.0])
    delta = _bits(orc, [0.25, 0.5, -0.125, -1.0])          # exactly representable sums
    new = orc.binop(orc.ADD, theta, delta)
    got = orc.edq(delta, theta, None, new, None)
    assert got == math.sqrt(0.25 ** 2 + 0.5 ** 2 + 0.125 ** 2 + 1.0)


def test_edq_zero_when_every_update_is_lost(orc):
    theta = _bits(orc, [200.0, -300.0, 1000.0])
    delta = _bits(orc, [0.1, 0.2, -0.5])
    new = orc.binop(orc.ADD, theta, delta)                 # F(200 (+) 0.1) = 200 (Sec. 3.1 Remark)
    assert np.array_equal(new, theta)
    assert orc.edq(delta, theta, None, new, None) == 0.0
    assert orc.edq(np.zeros(3, np.uint16), theta, None, new, None) == 0.0      # zero update: defined as 0


def test_edq_brute_force_and_expansion_form(orc):
    rng = np.random.default_rng(11)
    n = 500
    theta = H.np_round_f64_to_bf16(rng.standard_normal(n))
    dth = np.zeros(n, np.uint16)
    delta = H.np_round_f64_to_bf16(rng.standard_normal(n) * 1e-3)
    plain_new = orc.binop(orc.ADD, theta, delta)
    th1, dth1 = orc.grow(theta, dth, delta)

    def brute(t0, d0, t1, d1):
        s1 = Fraction(0)
        s2 = Fraction(0)
        for i in range(n):
            d = H.bf16_bits_to_fraction(delta[i])
            eff = (H.bf16_bits_to_fraction(t1[i]) + (H.bf16_bits_to_fraction(d1[i]) if d1 is not None else 0)) - \
                  (H.bf16_bits_to_fraction(t0[i]) + (H.bf16_bits_to_fraction(d0[i]) if d0 is not None else 0))
            s1 += d * eff
            s2 += d * d
        return float(s1) / math.sqrt(float(s2))

    e_plain = orc.edq(delta, theta, None, plain_new, None)
    e_mcf = orc.edq(delta, theta, dth, th1, dth1)
    assert abs(e_plain - brute(theta, None, plain_new, None)) <= 1e-12 * abs(e_plain)
    assert abs(e_mcf - brute(theta, dth, th1, dth1)) <= 1e-12 * abs(e_mcf)
    norm = math.sqrt(float(np.sum(H.u16_to_f64(delta) ** 2)))
    # the expansion keeps (almost) the whole update, plain bf16 loses a visible part of it
    assert abs(e_mcf - norm) < 1e-3 * norm
    assert abs(e_plain - norm) > 10 * abs(e_mcf - norm)
    # slices accumulate to the same totals
    acc = orc.EdqAccumulator()
    for lo in range(0, n, 123):
        hi = min(n, lo + 123)
        acc.add(delta[lo:hi].copy(), theta[lo:hi].copy(), dth[lo:hi].copy(), th1[lo:hi].copy(), dth1[lo:hi].copy())
    assert abs(acc.value() - e_mcf) <= 1e-12 * abs(e_mcf)
