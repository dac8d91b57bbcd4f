"""Pins for the oracle's two comparison strategies that share the Collage chain: plain bf16
(option A, Eq. 1) and Kahan-compensated bf16 (App. B "Kahan Summation", App. D "Equivalence"),
and for the lost-update counter (Def. 3.2; the imprecision percentage of the BERT case study).

Each is checked as a composition of primitives that are pinned on their own (single bf16
operations, Fast2Sum), against the behaviour the paper states, and by brute force.
"""
from fractions import Fraction

import numpy as np

import helpers as H
from paper_2405_03637_amd import workloads as W


def _state(n, seed, theta_std=0.02):
    theta = H.torch_to_u16(W.normal_bf16(n, theta_std, (seed, 200)))
    z = lambda: np.zeros(n, np.uint16)
    return dict(theta=theta, dtheta=z(), m=z(), v=z())


def _grads(n, seed, t, std=1e-3, mean=0.0):
    return H.torch_to_u16(W.normal_bf16(n, std, (seed, 201, t), mean=mean))


def test_plain_bf16_is_the_light_chain_with_one_rounded_addition(orc):
    """Option A differs from Collage-light only in line 13: theta <- F(theta + delta) (Eq. 1)."""
    n = 30_000
    hyper = (1e-2, 0.9, 0.95, 1e-8, 0.1)
    a, b = _state(n, 1), _state(n, 1)
    for t in range(1, 6):
        g = _grads(n, 1, t)
        da, db = np.empty(n, np.uint16), np.empty(n, np.uint16)
        theta_before = a["theta"].copy()
        orc.adamw_step(a["theta"], None, a["m"], a["v"], None, g, orc.BF16, hyper, t, delta_out=da)
        # the update depends on theta (weight decay), so feed light the same theta
        b["theta"][:] = theta_before
        b["dtheta"][:] = 0
        orc.adamw_step(b["theta"], b["dtheta"], b["m"], b["v"], None, g, orc.LIGHT, hyper, t, delta_out=db)
        assert np.array_equal(da, db) and np.array_equal(a["m"], b["m"]) and np.array_equal(a["v"], b["v"])
        assert np.array_equal(a["theta"], orc.binop(orc.ADD, theta_before, da))


def test_plain_bf16_loses_small_updates_collage_keeps_them(orc):
    """Sec. 3.2: when |delta| <= ulp(theta)/2 the bf16 parameter does not move at all; the expansion does."""
    n, steps = 4096, 200
    hyper = (2.0 ** -16, 0.9, 0.95, 1e-8, 0.0)
    plain, light = _state(n, 2, theta_std=1.0), _state(n, 2, theta_std=1.0)
    big = np.abs(H.u16_to_f64(plain["theta"])) > 0.01        # |delta| ~ 1.5e-5 < ulp/2 there
    th0 = plain["theta"].copy()
    for t in range(1, steps + 1):
        g = _grads(n, 2, t, mean=1e-3)
        orc.adamw_step(plain["theta"], None, plain["m"], plain["v"], None, g, orc.BF16, hyper, t)
        orc.adamw_step(light["theta"], light["dtheta"], light["m"], light["v"], None, g, orc.LIGHT, hyper, t)
    assert np.array_equal(plain["theta"][big], th0[big])
    moved = (H.u16_to_f64(light["theta"]) + H.u16_to_f64(light["dtheta"])) - H.u16_to_f64(th0)
    assert np.all(moved[big] < -0.5 * steps * hyper[0])      # steady positive gradients push theta down


def test_kahan_step_is_fast2sum_of_theta_and_compensated_update(orc):
    """App. D "Equivalence" (i): the Kahan variable is the error term of Fast2Sum(theta, u), u = F(delta + c)."""
    n = 30_000
    hyper = (1e-3, 0.9, 0.95, 1e-8, 0.1)
    st = _state(n, 3, theta_std=1.0)
    for t in range(1, 8):
        g = _grads(n, 3, t)
        d = np.empty(n, np.uint16)
        th0, c0 = st["theta"].copy(), st["dtheta"].copy()
        orc.adamw_step(st["theta"], st["dtheta"], st["m"], st["v"], None, g, orc.KAHAN, hyper, t, delta_out=d)
        u = orc.binop(orc.ADD, d, c0)
        x, y = orc.fast2sum(th0, u)
        assert np.array_equal(st["theta"], x) and np.array_equal(st["dtheta"], y)
        ok = np.abs(H.u16_to_f64(th0)) >= np.abs(H.u16_to_f64(u))
        exact = H.u16_to_f64(th0) + H.u16_to_f64(u)
        assert np.array_equal((H.u16_to_f64(x) + H.u16_to_f64(y))[ok], exact[ok])


def test_kahan_and_collage_light_follow_the_same_trajectory(orc):
    """App. D "Equivalence": with |theta| >> |delta| both keep theta_0 + sum(delta) to the resolution of the
    second component, and stay within a few of its ulps of each other."""
    n, steps = 8192, 300
    hyper = (2.0 ** -16, 0.9, 0.95, 1e-8, 0.1)
    k, l = _state(n, 4, theta_std=1.0), _state(n, 4, theta_std=1.0)
    th0 = H.u16_to_f64(k["theta"])
    big = np.abs(th0) > 0.05
    ideal = th0.copy()
    for t in range(1, steps + 1):
        g = _grads(n, 4, t, mean=5e-4)
        d = np.empty(n, np.uint16)
        orc.adamw_step(k["theta"], k["dtheta"], k["m"], k["v"], None, g, orc.KAHAN, hyper, t, delta_out=d)
        orc.adamw_step(l["theta"], l["dtheta"], l["m"], l["v"], None, g, orc.LIGHT, hyper, t)
        ideal += H.u16_to_f64(d)
    vk = H.u16_to_f64(k["theta"]) + H.u16_to_f64(k["dtheta"])
    vl = H.u16_to_f64(l["theta"]) + H.u16_to_f64(l["dtheta"])
    assert np.all(np.abs(vk - ideal)[big] <= steps * 2.0 ** -16 * np.abs(th0)[big])
    # weight decay makes the two delta streams differ slightly once the first components differ; the values agree
    assert np.median(np.abs(vk - vl)[big] / np.abs(ideal - th0)[big]) < 2.0 ** -6
    assert np.all(np.abs(vk - vl)[big] <= steps * 2.0 ** -15 * np.abs(th0)[big])


def test_lost_update_counter(orc):
    u = lambda vals: np.array([orc.B(v) for v in vals], np.uint16)
    theta = u([200.0, -300.0, 1.0, 4.0, 0.5])
    delta = u([0.1, 0.2, 0.25, 0.0, -2.0 ** -12])
    new = orc.binop(orc.ADD, theta, delta)
    acc = orc.EdqAccumulator()
    acc.add(delta, theta, None, new, None)
    # 200+0.1 and -300+0.2 are lost (Sec. 3.1 Remark), 1+0.25 is not, a zero update is not counted, 0.5-2^-12 is lost
    assert acc.lost.value == 3
    # with the expansion nothing is lost
    th1, d1 = orc.grow(theta, np.zeros(5, np.uint16), delta)
    acc = orc.EdqAccumulator()
    acc.add(delta, theta, np.zeros(5, np.uint16), th1, d1)
    assert acc.lost.value == 0
    # brute force on random data
    rng = np.random.default_rng(5)
    n = 3000
    th = H.np_round_f64_to_bf16(rng.standard_normal(n))
    de = H.np_round_f64_to_bf16(rng.standard_normal(n) * 10.0 ** rng.uniform(-6, -1, n))
    de[::17] = 0
    nw = orc.binop(orc.ADD, th, de)
    want = sum(1 for a, b, c in zip(th.tolist(), de.tolist(), nw.tolist())
               if H.bf16_bits_to_fraction(b) != 0 and H.bf16_bits_to_fraction(c) == H.bf16_bits_to_fraction(a))
    acc = orc.EdqAccumulator()
    acc.add(de, th, None, nw, None)
    assert acc.lost.value == want and 0 < want < n
    assert Fraction(want, n) > Fraction(1, 10)


def _ulp_arr(x):
    a = np.abs(x)
    _, e = np.frexp(a)
    e = e.astype(np.int64) - 1
    return np.where(a == 0, 2.0 ** -133, np.ldexp(1.0, (np.maximum(e, -126) - 7).astype(np.int32)))


def test_grow_on_two_sum_needs_no_ordering(orc):
    """App. C: TwoSum gives Fast2Sum's expansion without |a| >= |b|.  Grow built on it is therefore the same
    bits where Alg. 1's precondition |x| >= |a| holds, and keeps the Grow identity (the only loss is the
    rounding of y + v) where it does not -- e.g. parameters near zero, or v = 0 at the first step."""
    rng = np.random.default_rng(21)
    n = 1_000_000
    x = rng.choice(H.bf16_window(-8, 4), n)
    fx = H.u16_to_f64(x)
    y = H.np_round_f64_to_bf16(_ulp_arr(fx) * rng.uniform(-0.5, 0.5, n) * 0.99)
    # addends from 2^-20 of x up to 2^12 times x: half of them violate the precondition
    a = H.np_round_f64_to_bf16(fx * 2.0 ** rng.uniform(-20, 12, n) * rng.choice([-1.0, 1.0], n))
    fa, fy = H.u16_to_f64(a), H.u16_to_f64(y)
    x2, y2 = orc.grow_two_sum(x, y, a)
    xf, yf = orc.grow(x, y, a)
    pre = np.abs(fx) >= np.abs(fa)
    assert 0.3 < pre.mean() < 0.8
    nz = H.u16_to_f64(yf) != 0
    assert np.array_equal(x2[pre], xf[pre]) and np.array_equal(y2[pre & nz], yf[pre & nz])
    assert np.all(H.u16_to_f64(y2)[pre & ~nz] == 0)
    # identity for every ordering: u = RN(x+a), v = x+a-u exactly, t = RN(y+v); result = u + t exactly
    u = H.u16_to_f64(H.np_round_f64_to_bf16(fx + fa))
    v = (fx + fa) - u
    t_exact = fy + v
    t = H.u16_to_f64(H.np_round_f64_to_bf16(np.where(t_exact == 0, 0.0, t_exact)))
    got = H.u16_to_f64(x2) + H.u16_to_f64(y2)
    assert np.array_equal(got - (fx + fy + fa), t - t_exact)
    assert np.all(np.abs(H.u16_to_f64(y2)) <= _ulp_arr(H.u16_to_f64(x2)) / 2)
    # with Fast2Sum the identity does fail somewhere outside the precondition
    gotf = H.u16_to_f64(xf) + H.u16_to_f64(yf)
    assert np.any((gotf - (fx + fy + fa))[~pre] != (t - t_exact)[~pre])


def test_step_with_two_sum_grow(orc):
    """The flagged step equals the plain one while the preconditions hold, and differs only through Grow."""
    n = 20_000
    hyper = (1e-3, 0.9, 0.999, 1e-8, 0.1)
    a = dict(_state(n, 8, theta_std=1.0), dv=np.zeros(n, np.uint16))
    b = {k: v.copy() for k, v in a.items()}
    ema = np.zeros(n)
    for t in range(1, 30):
        g = _grads(n, 8, t)
        orc.adamw_step(a["theta"], a["dtheta"], a["m"], a["v"], a["dv"], g, orc.PLUS, hyper, t)
        orc.adamw_step(b["theta"], b["dtheta"], b["m"], b["v"], b["dv"], g, orc.PLUS | orc.GROW_TWOSUM, hyper, t)
        assert np.array_equal(a["m"], b["m"])
        ema = 0.999 * ema + 0.001 * H.u16_to_f64(g) ** 2
    # |theta| ~ 1 >> |delta| ~ 1e-3 except for the few elements near zero: nearly all trajectories coincide
    assert np.mean(a["theta"] == b["theta"]) > 0.99
    # v is young here (v ~ t * 0.001 g^2), so a large gradient often exceeds it and breaks Fast2Sum's ordering;
    # the TwoSum flavour follows the true average at least as well
    ea = np.abs(H.u16_to_f64(a["v"]) + H.u16_to_f64(a["dv"]) - ema) / ema
    eb = np.abs(H.u16_to_f64(b["v"]) + H.u16_to_f64(b["dv"]) - ema) / ema
    assert eb.max() < 2.0 ** -7 and np.median(eb) < 2.0 ** -9
    assert eb.mean() <= ea.mean() * 1.001


def test_mcf_sgd(orc):
    """MCF-SGD with momentum (Sec. 1: "extensions to SGD are straight-forward"): checked as a composition of
    pinned primitives, against torch's fp64 SGD (momentum, no decay) and against the closed form of pure decay."""
    import torch
    n, steps = 10_000, 80
    lr, mu = 2.0 ** -14, 0.9
    st = _state(n, 9, theta_std=1.0)
    th0 = H.u16_to_f64(st["theta"])
    p = torch.nn.Parameter(torch.tensor(th0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=lr, momentum=mu)
    b1 = np.full(n, orc.B(mu), np.uint16)
    plain = st["theta"].copy()
    for t in range(1, steps + 1):
        g = _grads(n, 9, t, std=1.0, mean=0.5)
        d = np.empty(n, np.uint16)
        th_b, dth_b, m_b = st["theta"].copy(), st["dtheta"].copy(), st["m"].copy()
        orc.adamw_step(st["theta"], st["dtheta"], st["m"], None, None, g, orc.SGD, (lr, mu, 0.0, 0.0, 0.0), t, delta_out=d)
        # composition of single operations and Grow
        assert np.array_equal(st["m"], orc.binop(orc.ADD, orc.binop(orc.MUL, b1, m_b), g))
        gx, gy = orc.grow(th_b, dth_b, d)
        assert np.array_equal(st["theta"], gx) and np.array_equal(st["dtheta"], gy)
        plain = orc.binop(orc.ADD, plain, d)
        p.grad = torch.tensor(H.u16_to_f64(g), dtype=torch.float64)
        opt.step()
    ref = p.detach().numpy()
    got = H.u16_to_f64(st["theta"]) + H.u16_to_f64(st["dtheta"])
    moved = np.abs(ref - th0)
    big = np.abs(th0) > 0.3
    assert np.median(moved) > 0.01
    # the momentum buffer carries 8 bits: a few 2^-8 of the distance travelled, plus the expansion's resolution
    assert np.all(np.abs(got - ref)[big] <= 0.03 * moved[big] + steps * 2.0 ** -16 * np.abs(th0)[big])
    # every single update is below half an ulp of theta there, so plain bf16 accumulation is far worse
    assert np.median(np.abs(H.u16_to_f64(plain) - ref)[big]) > 10 * np.median(np.abs(got - ref)[big])
    # pure decay: zero gradients
    st = _state(n, 10, theta_std=1.0)
    th0 = H.u16_to_f64(st["theta"])
    z = np.zeros(n, np.uint16)
    for t in range(1, 101):
        orc.adamw_step(st["theta"], st["dtheta"], st["m"], None, None, z, orc.SGD, (1e-3, 0.9, 0.0, 0.0, 0.1), t)
    got = H.u16_to_f64(st["theta"]) + H.u16_to_f64(st["dtheta"])
    want = th0 * (1 - 1e-3 * 0.1) ** 100
    assert np.all(np.abs(got - want) <= 0.012 * np.abs(th0 - want) + 100 * 2.0 ** -17 * np.abs(th0))
    assert not st["m"].any()
