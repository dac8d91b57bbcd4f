"""The Collage step in EXACT rational arithmetic, one round-to-nearest-even per operation.

Test infrastructure, independent of the oracle and of the GPU library: operands are bf16 bit patterns,
every operation forms its exact rational result with Python's Fraction and rounds it ONCE to bf16 by
searching the table of all bf16 values (helpers.nearest_bf16) -- no fp32 anywhere.  For + - * / and sqrt
of bf16 operands that is what F(a o b) must give (rounding through fp32 first cannot change the result:
24 >= 2*8+2), so the oracle's fp32-then-round route and this route have to agree bit for bit through
whole steps.  Finite inputs only; zero results carry IEEE's sign.
"""
import math
from fractions import Fraction

import helpers as H

val = H.bf16_bits_to_fraction
SIGN = 0x8000


def _is_zero(h):
    return (h & 0x7FFF) == 0


def add(a, b):
    x = val(a) + val(b)
    if x == 0:      # exact cancellation gives +0 under round-to-nearest, unless both operands are -0
        return SIGN if (_is_zero(a) and _is_zero(b) and (a & SIGN) and (b & SIGN)) else 0
    return H.nearest_bf16(x)


def sub(a, b):
    return add(a, b ^ SIGN)


def mul(a, b):
    x = val(a) * val(b)
    if x == 0:
        return (a ^ b) & SIGN
    return H.nearest_bf16(x)


def div(a, b):
    assert not _is_zero(b)
    x = val(a) / val(b)
    if x == 0:
        return (a ^ b) & SIGN
    return H.nearest_bf16(x)


def fms(a, b, c):
    """F(a*b - c), the product exact (Alg. 6)."""
    x = val(a) * val(b) - val(c)
    if x == 0:
        return 0
    return H.nearest_bf16(x)


def sqrt(a):
    x = val(a)
    assert x >= 0
    if x == 0:
        return a
    g = H.nearest_bf16(Fraction(math.sqrt(float(x))))     # a guess; the bracket below decides
    while True:
        c = val(g)
        lo = (c + val(g - 1)) / 2
        hi = (c + val(g + 1)) / 2
        if x < lo * lo:
            g -= 1
        elif x > hi * hi:
            g += 1
        else:
            assert lo * lo != x and hi * hi != x          # the root of a bf16 is never a rounding tie
            return g


def fast2sum(a, b):                      # Thm 4.1
    x = add(a, b)
    return x, sub(b, sub(x, a))


def two_sum(a, b):                       # Alg. 3
    x = add(a, b)
    bv = sub(x, a)
    av = sub(x, bv)
    return x, add(sub(a, av), sub(b, bv))


def grow(x, y, a, twosum=False):         # Alg. 1
    s = two_sum if twosum else fast2sum
    u, w = s(x, a)
    return s(u, add(y, w))


def mul_expansion(a1, a2, b1, b2):       # Alg. 8 with Alg. 6
    x = mul(a1, b1)
    e = add(fms(a1, b1, x), add(mul(a1, b2), mul(a2, b1)))
    return fast2sum(x, e)


def scalars(hyper, t):
    """fp64 formulas, one rounding each (App. D); exact rationals of the double inputs."""
    lr, b1, b2, eps, wd = (Fraction(x) for x in hyper)
    B = lambda x: H.nearest_bf16(x) if x != 0 else 0
    b2h = B(b2)
    # 1 - beta^t is formed in fp64 by the implementations; for the t used in the tests beta^t is taken
    # with float pow and the subtraction is exact in rationals, then rounded once to fp64 by float()
    bc = lambda b: B(Fraction(1.0 - float(b) ** t))
    return dict(b1=B(b1), c1=B(Fraction(1.0 - float(b1))), b2=b2h, b2l=B(b2 - val(b2h)), c2=B(Fraction(1.0 - float(b2))),
                bc1=bc(b1), bc2=bc(b2), e=B(eps), lam=B(wd), na=B(-lr))


def adamw_element(st, g, variant, s, twosum=False):
    """st: dict theta, dtheta, m, v, dv of bit patterns (one element).  variant: light, plus, bf16, kahan, sgd.
    Returns delta; st is updated.  The sequence is Alg. 2 lines 8-13 as read by this build."""
    th, dth, m, v, dv = st["theta"], st["dtheta"], st["m"], st["v"], st["dv"]
    if variant == "sgd":
        m1 = add(mul(s["b1"], m), g)
        delta = mul(s["na"], add(m1, mul(s["lam"], th)))
        st["theta"], st["dtheta"] = grow(th, dth, delta)
        st["m"] = m1
        return delta
    m1 = add(mul(s["b1"], m), mul(s["c1"], g))
    inc = mul(s["c2"], mul(g, g))
    if variant == "plus":
        X, E = mul_expansion(s["b2"], s["b2l"], v, dv)
        v1, dv1 = grow(X, E, inc, twosum)
    else:
        v1, dv1 = add(mul(s["b2"], v), inc), dv
    mh, vh = div(m1, s["bc1"]), div(v1, s["bc2"])
    dn = add(sqrt(vh), s["e"])
    delta = mul(s["na"], add(div(mh, dn), mul(s["lam"], th)))
    if variant == "bf16":
        th1, dth1 = add(th, delta), dth
    elif variant == "kahan":
        u = add(delta, dth)
        th1 = add(th, u)
        dth1 = sub(u, sub(th1, th))
    else:
        th1, dth1 = grow(th, dth, delta, twosum)
    st.update(theta=th1, dtheta=dth1, m=m1, v=v1, dv=dv1)
    return delta
