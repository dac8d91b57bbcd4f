"""Pins for the WIRING of the oracle's step: which operand feeds which operation, in which order.

The single operations F(a o b) and the expansion primitives are pinned on their own (exhaustively, against
exact arithmetic and the paper's printed values).  What those pins cannot see is a mistake in how Alg. 2's
lines are put together from them -- an association the paper leaves open read differently in one place, a
flag that is accepted and then ignored, a line fed the old value of a moment.  Here every variant of the
step is rebuilt from the pinned single operations, in the sequence this build reads out of Alg. 2 and
App. D (every arithmetic symbol rounded on its own; (1-beta2) * (g*g); decay lambda*theta on the first
component, summed with the ratio and then scaled by -alpha once; bias corrections on the new moments; first
components only in lines 10-12), on states that break Grow's ordering assumption for a fair share of the
elements so that the Fast2Sum and TwoSum flavours really differ.  Also: every scalar is cast to the
component format in ONE rounding from fp64, and both steps of the TwoSum-based Grow are error-free for
every FP8 operand triple.
"""
import numpy as np
import pytest

import helpers as H

FMTS = [0, 1, 2, 3]      # bf16, fp16, FP8 E5M2, FP8 E4M3


def _patterns(orc, fmt, n, rng, lo_exp, hi_exp, signed=True):
    """n finite patterns of the format with magnitudes spread log-uniformly over [2^lo_exp, 2^hi_exp)."""
    mag = 2.0 ** rng.uniform(lo_exp, hi_exp, n)
    if signed:
        mag *= rng.choice([-1.0, 1.0], n)
    return orc.R_array(mag.astype(np.float32), fmt=fmt)


def _second_component(orc, fmt, first, rng):
    """A second component below half a unit in the last place of the first."""
    f = orc.widen_array(first, fmt=fmt).astype(np.float64)
    return orc.R_array((f * 2.0 ** -12 * rng.uniform(-1, 1, f.size)).astype(np.float32), fmt=fmt)


def _splat(bits, n):
    return np.full(n, bits, np.uint16)


def _setup(orc, fmt, n, seed):
    rng = np.random.default_rng(seed)
    wide = fmt < 2                       # the 8-bit formats have little range: keep everything near 1
    theta = _patterns(orc, fmt, n, rng, -6 if wide else -3, 1 if wide else 1)
    theta[: n // 4] = _patterns(orc, fmt, n // 4, rng, -14 if wide else -6, -9 if wide else -4)   # near zero: |theta| < |delta|
    dtheta = _second_component(orc, fmt, theta, rng)
    k = n // 2
    # some second components that OVERLAP the first (not what Grow leaves behind, but nothing forbids a
    # caller's state from holding them): only there can "lambda * theta" be told from "lambda * (theta + dtheta)"
    dtheta[k: k + n // 8] = orc.binop(orc.MUL, theta[k: k + n // 8], np.full(n // 8, orc.B(0.0625 if wide else 0.5, fmt=fmt), np.uint16), fmt=fmt)
    st = dict(theta=theta, dtheta=dtheta,
              m=_patterns(orc, fmt, n, rng, -5 if wide else -3, -1),
              v=_patterns(orc, fmt, n, rng, -12 if wide else -5, -2, signed=False))
    st["dv"] = _second_component(orc, fmt, st["v"], rng)
    g = _patterns(orc, fmt, n, rng, -6 if wide else -3, 0)
    hyper = (2.0 ** -6 * 1.3, 0.9, 0.95, 2.0 ** -7, 0.3) if wide else (0.09375, 0.625, 0.8125, 2.0 ** -6, 0.375)
    return st, g, hyper


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("base,flags", [("LIGHT", 0), ("LIGHT", "GROW_TWOSUM"), ("PLUS", 0), ("PLUS", "GROW_TWOSUM"),
                                        ("BF16", 0), ("KAHAN", 0), ("LIGHT", "EPS_INSIDE_SQRT")])
def test_adamw_step_is_the_stated_sequence_of_single_operations(orc, fmt, base, flags):
    n, t = 60_000, 3
    st, g, hyper = _setup(orc, fmt, n, 400 + fmt)
    variant = getattr(orc, base) | (getattr(orc, flags) if flags else 0)
    s = {k: _splat(b, n) for k, b in orc.scalars(*hyper, t, fmt=fmt).items()}
    op = lambda code, a, b=None: orc.binop(code, a, b, fmt=fmt)
    ADD, SUB, MUL, DIV, SQRT = orc.ADD, orc.SUB, orc.MUL, orc.DIV, orc.SQRT
    twosum = flags == "GROW_TWOSUM"
    grow = (lambda x, y, a: orc.prim(orc.GROW2, x, y, a, fmt=fmt)) if twosum else (lambda x, y, a: orc.prim(orc.GROW, x, y, a, fmt=fmt))

    m1 = op(ADD, op(MUL, s["b1"], st["m"]), op(MUL, s["c1"], g))                    # line 8
    inc = op(MUL, s["c2"], op(MUL, g, g))                                           # line 9: (1-beta2) * (g*g)
    if base == "PLUS":
        X, E = orc.prim(orc.MULX, s["b2"], s["b2l"], st["v"], st["dv"], fmt=fmt)
        v1, dv1 = grow(X, E, inc)
    else:
        v1, dv1 = op(ADD, op(MUL, s["b2"], st["v"]), inc), None
    mh, vh = op(DIV, m1, s["bc1"]), op(DIV, v1, s["bc2"])                           # lines 10-11, on the new moments
    dn = op(SQRT, op(ADD, vh, s["e"])) if flags == "EPS_INSIDE_SQRT" else op(ADD, op(SQRT, vh), s["e"])
    delta = op(MUL, s["na"], op(ADD, op(DIV, mh, dn), op(MUL, s["lam"], st["theta"])))     # line 12
    if base == "BF16":
        th1, dth1 = op(ADD, st["theta"], delta), st["dtheta"]                       # Eq. 1; the second array is not touched
    elif base == "KAHAN":
        u = op(ADD, delta, st["dtheta"])
        th1 = op(ADD, st["theta"], u)
        dth1 = op(SUB, u, op(SUB, th1, st["theta"]))
    else:
        th1, dth1 = grow(st["theta"], st["dtheta"], delta)                          # line 13

    got = {k: v.copy() for k, v in st.items()}
    d = np.empty(n, np.uint16)
    orc.adamw_step(got["theta"], got["dtheta"], got["m"], got["v"], got["dv"] if base == "PLUS" else None, g,
                   variant | orc.step_flag(fmt), hyper, t, delta_out=d)
    for name, want in (("delta", delta), ("m", m1), ("v", v1), ("theta", th1), ("dtheta", dth1)):
        have = d if name == "delta" else got[name]
        bad = np.flatnonzero(have != want)
        assert bad.size == 0, f"{name}: {bad.size} of {n} differ, first at {bad[0]}"
    if base == "PLUS":
        assert np.array_equal(got["dv"], dv1)

    # the data can tell the readings apart: each alternative changes a fair share of the results
    share = lambda a, b: float(np.mean(a != b))
    assert share(inc, op(MUL, op(MUL, s["c2"], g), g)) > 0.02                                           # (c2*g)*g
    full = op(ADD, st["theta"], st["dtheta"])
    alt = op(MUL, s["na"], op(ADD, op(DIV, mh, dn), op(MUL, s["lam"], full)))
    distributed = op(ADD, op(MUL, s["na"], op(DIV, mh, dn)), op(MUL, s["na"], op(MUL, s["lam"], st["theta"])))
    assert share(delta, distributed) > 0.02
    assert share(delta, alt) > 0.01                                        # decay on the whole value theta + dtheta
    assert share(op(DIV, m1, s["bc1"]), op(DIV, st["m"], s["bc1"])) > 0.5
    if base in ("LIGHT", "PLUS"):
        other = (lambda x, y, a: orc.prim(orc.GROW, x, y, a, fmt=fmt)) if twosum else (lambda x, y, a: orc.prim(orc.GROW2, x, y, a, fmt=fmt))
        ox, oy = other(st["theta"], st["dtheta"], delta)
        assert share(dth1, oy) + share(th1, ox) > 0.01            # Fast2Sum and TwoSum flavours differ near zero
        if base == "PLUS":
            ox, oy = other(X, E, inc)
            assert share(dv1, oy) + share(v1, ox) > 0.001


@pytest.mark.parametrize("fmt", FMTS)
def test_sgd_step_is_the_stated_sequence_of_single_operations(orc, fmt):
    """m <- mu*m + g ; delta <- -alpha*(m + lambda*theta) on the NEW m ; (theta, dtheta) <- Grow(., delta)."""
    n, t = 60_000, 5
    st, g, hyper = _setup(orc, fmt, n, 420 + fmt)
    s = {k: _splat(b, n) for k, b in orc.scalars(*hyper, t, fmt=fmt).items()}
    op = lambda code, a, b=None: orc.binop(code, a, b, fmt=fmt)
    m1 = op(orc.ADD, op(orc.MUL, s["b1"], st["m"]), g)
    delta = op(orc.MUL, s["na"], op(orc.ADD, m1, op(orc.MUL, s["lam"], st["theta"])))
    th1, dth1 = orc.prim(orc.GROW, st["theta"], st["dtheta"], delta, fmt=fmt)
    got = {k: v.copy() for k, v in st.items()}
    d = np.empty(n, np.uint16)
    orc.adamw_step(got["theta"], got["dtheta"], got["m"], None, None, g, orc.SGD | orc.step_flag(fmt), hyper, t, delta_out=d)
    assert np.array_equal(d, delta) and np.array_equal(got["m"], m1)
    assert np.array_equal(got["theta"], th1) and np.array_equal(got["dtheta"], dth1)
    stale = op(orc.MUL, s["na"], op(orc.ADD, st["m"], op(orc.MUL, s["lam"], st["theta"])))
    assert np.mean(stale != delta) > 0.5


# ------------------------------------------------------------------ scalars: one rounding from fp64
def _just_above_a_tie(fmt_bits):
    """1 + half a unit in the last place + 2^-40: rounds up in one rounding; through fp32 the 2^-40 is lost
    first, the rest is an exact tie, and ties-to-even rounds DOWN to 1."""
    return 1.0 + 2.0 ** -(fmt_bits + 1) + 2.0 ** -40


@pytest.mark.parametrize("fmt,mbits,one,next_up", [(0, 7, 0x3F80, 0x3F81), (1, 10, 0x3C00, 0x3C01), (2, 2, 0x3C, 0x3D), (3, 3, 0x38, 0x39)])
def test_scalars_are_cast_in_one_rounding(orc, fmt, mbits, one, next_up):
    x = _just_above_a_tie(mbits)
    assert orc.R(np.float32(x), fmt=fmt) == one and orc.B(x, fmt=fmt) == next_up        # the two routes do differ here
    sign = 0x8000 if fmt < 2 else 0x80
    half = {0: 0x3F00, 1: 0x3800, 2: 0x38, 3: 0x30}[fmt]
    s = orc.scalars(x, 0.5, 0.5, x, x, 1, fmt=fmt)
    assert s["e"] == next_up and s["lam"] == next_up and s["na"] == (next_up | sign)
    # beta = x/2 (< 1): b = next_up at half the scale
    b = x / 2
    s = orc.scalars(1e-3, b, b, 1e-8, 0.0, 1, fmt=fmt)
    want_b = orc.B(b, fmt=fmt)
    assert want_b == next_up - (1 << mbits) and s["b1"] == want_b and s["b2"] == want_b
    assert s["c1"] == orc.B(1.0 - b, fmt=fmt) == s["c2"] == s["bc1"] == s["bc2"]
    assert s["c1"] != orc.B(1.0 - float(orc.widen(want_b, fmt=fmt)), fmt=fmt)          # taken from beta itself, not from its rounding
    assert orc.B(0.5, fmt=fmt) == half
    # the second component of beta2 is the rounding of what the first left over, computed exactly
    left = b - float(orc.widen(want_b, fmt=fmt))
    assert s["b2l"] == orc.B(left, fmt=fmt) and left != 0.0


# ------------------------------------------------------------------ Grow on TwoSum, every FP8 triple
@pytest.mark.parametrize("fmt", [2, 3])
def test_grow_on_two_sum_is_error_free_in_both_steps_for_every_fp8_triple(orc, fmt):
    """(u, w) = TwoSum(x, a) and (x', y') = TwoSum(u, F(y + w)) are both error-free for every ordering of
    their operands (App. C), so u + w = x + a and x' + y' = u + F(y + w) exactly -- for all 2^24 (x, y, a),
    wherever nothing overflows.  A Fast2Sum in either place breaks this for many triples."""
    codes = np.arange(256, dtype=np.uint16)
    val = orc.widen_array(codes, fmt=fmt).astype(np.float64)
    top = np.nanmax(np.where(np.isfinite(val), np.abs(val), 0))
    finite = codes[np.isfinite(val)]
    x = np.repeat(finite, finite.size)
    a = np.tile(finite, finite.size)
    u, w = orc.two_sum(x, a, fmt=fmt)
    fu, fw = val[u], val[w]
    ok_first = np.isfinite(fu) & np.isfinite(fw) & (np.abs(val[x] + val[a]) < top)     # next to the top an intermediate overflows
    assert ok_first.mean() > 0.9
    assert np.array_equal((fu + fw)[ok_first], (val[x] + val[a])[ok_first])
    checked = broken_by_fast2sum = 0
    for y in finite:
        yy = np.full(x.size, y, np.uint16)
        gx, gy = orc.prim(orc.GROW2, x, yy, a, fmt=fmt)
        t = orc.binop(orc.ADD, yy, w, fmt=fmt)
        ft, fgx, fgy = val[t], val[gx], val[gy]
        ok = ok_first & np.isfinite(ft) & np.isfinite(fgx) & np.isfinite(fgy) & (np.abs(fu + ft) < top)
        assert np.array_equal((fgx + fgy)[ok], (fu + ft)[ok]), f"y pattern {y:#04x}"
        checked += int(ok.sum())
        fx2, fy2 = orc.fast2sum(u, t, fmt=fmt)
        with np.errstate(invalid="ignore"):
            broken_by_fast2sum += int(np.sum((val[fx2] + val[fy2])[ok] != (fu + ft)[ok]))
    assert checked > 0.8 * finite.size ** 3
    assert broken_by_fast2sum > 1000


# ------------------------------------------------------------------ option D, operation by operation
def test_fp32_master_step_is_the_stated_sequence_of_ieee_single_operations(orc):
    """The fp32-master baseline (option D): AdamW's formulas with one IEEE binary32 operation per arithmetic
    symbol, scalars cast once from fp64 (1-beta and 1-beta^t formed in fp64 first), decay taken on the fp32
    master weight, the bf16 parameter refreshed by one rounding of the new master weight.  Rebuilt here with
    numpy's float32 array arithmetic (IEEE +, *, / and a correctly rounded sqrt), bit for bit, over several
    steps from a state with history; each alternative wiring is shown to differ on this data."""
    n = 50_000
    rng = np.random.default_rng(77)
    hyper = (1e-3, 0.9, 0.999, 1e-8, 0.1)
    lr, b1, b2, eps, wd = hyper
    f = np.float32
    master = rng.normal(0, 0.5, n).astype(f)
    theta = orc.R_array(master)
    m = rng.normal(0, 1e-3, n).astype(f)
    v = (rng.normal(0, 1e-3, n) ** 2).astype(f)
    ref = dict(master=master.copy(), m=m.copy(), v=v.copy())
    alt_seen = dict(decay_on_theta16=0, c_from_float=0, distributed=0)
    for t in range(3, 9):
        g16 = orc.R_array(rng.normal(0, 1e-3, n).astype(f))
        g = H.u16_to_f32(g16)
        sb1, sc1, sb2, sc2 = f(b1), f(1.0 - b1), f(b2), f(1.0 - b2)
        bc1, bc2 = f(1.0 - b1 ** t), f(1.0 - b2 ** t)
        se, slam, sna = f(eps), f(wd), f(-lr)
        m1 = sb1 * ref["m"] + sc1 * g
        v1 = sb2 * ref["v"] + sc2 * (g * g)
        ratio = (m1 / bc1) / (np.sqrt(v1 / bc2) + se)
        delta = sna * (ratio + slam * ref["master"])
        assert m1.dtype == v1.dtype == delta.dtype == np.float32
        # alternatives, on the same inputs
        theta16 = H.u16_to_f32(orc.R_array(ref["master"]))
        alt_seen["decay_on_theta16"] += int(np.sum(sna * (ratio + slam * theta16) != delta))
        alt_seen["c_from_float"] += int(np.sum(sb2 * ref["v"] + (f(1.0) - sb2) * (g * g) != v1))
        alt_seen["distributed"] += int(np.sum(sna * ratio + sna * (slam * ref["master"]) != delta))
        ref["master"] = ref["master"] + delta
        ref["m"], ref["v"] = m1, v1
        orc.fp32mw_step(theta, master, m, v, g16, hyper, t)
        for name, have in (("master", master), ("m", m), ("v", v)):
            assert np.array_equal(have.view(np.uint32), ref[name].view(np.uint32)), f"step {t}: {name}"
        assert np.array_equal(theta, orc.R_array(ref["master"])), f"step {t}: theta"
    assert all(c > n // 100 for c in alt_seen.values()), alt_seen
