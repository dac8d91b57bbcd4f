"""The oracle's steps against an independent evaluation in exact rational arithmetic (tests/exact_chain.py):
every operation's exact result rounded once to bf16 by table search, no fp32 involved, written in another
language with other data structures.  Agreement over whole multi-step trajectories pins the oracle's
arithmetic (F through fp32 equals one rounding of the exact result, also for the divisions, the root and
the fused multiply-subtract) and its wiring at once."""
import numpy as np
import pytest

import exact_chain as X
import helpers as H


def _draw(rng, n, lo, hi, signed=True):
    mag = 2.0 ** rng.uniform(lo, hi, n) * (rng.choice([-1.0, 1.0], n) if signed else 1.0)
    return H.np_round_f64_to_bf16(mag)


@pytest.mark.parametrize("variant,code,twosum", [("light", 0, False), ("plus", 1, False), ("bf16", 2, False), ("kahan", 3, False),
                                                 ("sgd", 4, False), ("light", 0, True), ("plus", 1, True)])
def test_steps_in_exact_rational_arithmetic(orc, variant, code, twosum):
    n, steps = 400, 4
    rng = np.random.default_rng(500 + code + 10 * twosum)
    hyper = (1.3e-3, 0.9, 0.999, 1e-8, 0.1)
    theta = _draw(rng, n, -8, 1)
    theta[: n // 4] = _draw(rng, n // 4, -16, -10)            # near zero: Grow's ordering assumption fails there
    st = dict(theta=theta, dtheta=np.zeros(n, np.uint16), m=_draw(rng, n, -12, -6), v=_draw(rng, n, -22, -12, signed=False),
              dv=np.zeros(n, np.uint16))
    mine = [{k: int(a[i]) for k, a in st.items()} for i in range(n)]
    theta0 = theta.copy()
    flags = orc.GROW_TWOSUM if twosum else 0
    for t in range(1, steps + 1):
        g = _draw(rng, n, -14, -5)
        d = np.empty(n, np.uint16)
        orc.adamw_step(st["theta"], st["dtheta"] if variant != "bf16" else None, st["m"], st["v"] if variant != "sgd" else None,
                       st["dv"] if variant == "plus" else None, g, code | flags, hyper, t, delta_out=d)
        s = X.scalars(hyper, t)
        assert s == orc.scalars(*hyper, t)
        for i in range(n):
            delta = X.adamw_element(mine[i], int(g[i]), variant, s, twosum)
            assert delta == int(d[i]), f"step {t} element {i}: delta {delta:#06x} against the oracle's {int(d[i]):#06x}"
            for k in ("theta", "dtheta", "m", "v", "dv"):
                assert mine[i][k] == int(st[k][i]), f"step {t} element {i} {k}: {mine[i][k]:#06x} against {int(st[k][i]):#06x}"
    moved = sum(mine[i]["theta"] != int(theta0[i]) or mine[i]["dtheta"] != 0 for i in range(n))
    assert moved > (0.5 if variant == "bf16" else 0.9) * n        # plain bf16 loses the small updates (Sec. 3.2)


@pytest.mark.parametrize("variant,code", [("light", 0), ("plus", 1)])
def test_steps_among_subnormal_moments_in_exact_rational_arithmetic(orc, variant, code):
    """The same with moments and gradients so small that products, quotients and the root's operand are
    subnormal or underflow to zero: the oracle's fp32 intermediates are subnormal there, the exact route has
    no such thing, and the two must still agree."""
    n, steps = 300, 3
    rng = np.random.default_rng(520 + code)
    hyper = (1.3e-3, 0.9, 0.95, 1e-8, 0.1)
    st = dict(theta=_draw(rng, n, -8, 1), dtheta=np.zeros(n, np.uint16), m=_draw(rng, n, -133, -120),
              v=_draw(rng, n, -133, -118, signed=False), dv=np.zeros(n, np.uint16))
    mine = [{k: int(a[i]) for k, a in st.items()} for i in range(n)]
    for t in range(1, steps + 1):
        g = _draw(rng, n, -70, -58)
        g[::7] = 0
        d = np.empty(n, np.uint16)
        orc.adamw_step(st["theta"], st["dtheta"], st["m"], st["v"], st["dv"] if variant == "plus" else None, g, code, hyper, t, delta_out=d)
        s = X.scalars(hyper, t)
        for i in range(n):
            delta = X.adamw_element(mine[i], int(g[i]), variant, s)
            assert delta == int(d[i]), f"step {t} element {i}: delta"
            for k in ("theta", "dtheta", "m", "v", "dv"):
                assert mine[i][k] == int(st[k][i]), f"step {t} element {i} {k}: {mine[i][k]:#06x} against {int(st[k][i]):#06x}"
    assert float(np.mean((st["v"] & 0x7F80) == 0)) > 0.1     # a good share of the second moments is subnormal or zero
