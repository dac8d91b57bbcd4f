"""Pins for the oracle's AdamW chains (Alg. 2, light and plus) and the fp32-master baseline (option D).

The paper prints no worked AdamW step, so bit patterns of the chain are not pinned by a printed value.
What IS pinned here: the scalars (Table 2, App. D), the closed form of the first step, the trajectory of a
textbook fp64 AdamW (torch.optim.AdamW on float64, fed the same bf16 gradients), the behaviour the paper
states for beta2 = 0.999 (Sec. 4.2: plain bf16 v only grows; the expansion follows the true average),
and the accumulation identity of Grow.  Each is chosen so that a dropped term, a wrong sign, a misplaced
epsilon, a missing bias correction or swapped Mul operands fails.
"""
import numpy as np
import pytest
import torch

import helpers as H
from paper_2405_03637_amd import workloads as W


def _state(n, seed, theta_std=0.02, plus=False):
    theta = H.torch_to_u16(W.normal_bf16(n, theta_std, (seed, 100)))
    z = lambda: np.zeros(n, np.uint16)
    return dict(theta=theta, dtheta=z(), m=z(), v=z(), dv=z() if plus else None)


def _grads(n, seed, step, std=1e-3, mean=0.0):
    return H.torch_to_u16(W.normal_bf16(n, std, (seed, 101, step), mean=mean))


def _run(orc, st, variant, hyper, steps, gradfn, deltas=None):
    n = st["theta"].size
    for t in range(1, steps + 1):
        g = gradfn(t)
        d = np.empty(n, np.uint16) if deltas is not None else None
        orc.adamw_step(st["theta"], st["dtheta"], st["m"], st["v"], st["dv"], g, variant, hyper, t, delta_out=d)
        if deltas is not None:
            deltas.append(d)


def _torch_adamw_fp64(theta0, grads, hyper):
    lr, b1, b2, eps, wd = hyper
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
    st = opt.state[p]
    return p.detach().numpy().copy(), st["exp_avg"].numpy().copy(), st["exp_avg_sq"].numpy().copy()


# ------------------------------------------------------------------ scalars
def test_scalars(orc):
    s = orc.scalars(3e-4, 0.9, 0.95, 1e-8, 0.1, 1)
    w = orc.widen
    assert s["b1"] == H.nearest_bf16(0.9) and s["c1"] == H.nearest_bf16(1 - 0.9)
    assert s["b2"] == H.nearest_bf16(0.95) and s["c2"] == H.nearest_bf16(1 - 0.95)
    assert s["bc1"] == H.nearest_bf16(1 - 0.9) and s["bc2"] == H.nearest_bf16(1 - 0.95)       # t = 1
    assert s["e"] == H.nearest_bf16(1e-8) and s["lam"] == H.nearest_bf16(0.1)
    assert s["na"] == (H.nearest_bf16(3e-4) | 0x8000)
    assert s["b2l"] == H.nearest_bf16(0.95 - w(s["b2"]))
    s7 = orc.scalars(3e-4, 0.9, 0.999, 1e-8, 0.1, 7)
    assert s7["bc1"] == H.nearest_bf16(1 - 0.9 ** 7) and s7["bc2"] == H.nearest_bf16(1 - 0.999 ** 7)
    assert w(s7["b2"]) == 1.0 and round(w(s7["b2l"]), 3) == -0.001                           # Table 2
    # bias corrections tend to exactly 1.0
    assert w(orc.scalars(3e-4, 0.9, 0.95, 1e-8, 0.1, 10_000)["bc2"]) == 1.0


# ------------------------------------------------------------------ first step: closed form
@pytest.mark.parametrize("variant", [0, 1])
def test_first_step_closed_form(orc, variant):
    """t = 1, m = v = 0: m_hat = g and v_hat = g^2 up to a few bf16 roundings, so
    delta = -lr * ( g/(|g|+eps) + wd*theta ).  eps is chosen comparable to |g| so that its placement
    (outside the square root) and the bias corrections are visible; wd*theta is comparable to the ratio."""
    n = 4096
    hyper = (1e-2, 0.9, 0.95, 1e-3, 0.5)
    st = _state(n, 1, theta_std=1.0, plus=bool(variant))
    theta0 = H.u16_to_f64(st["theta"])
    g = _grads(n, 1, 1, std=2e-3)
    deltas = []
    _run(orc, st, variant, hyper, 1, lambda t: g, deltas)
    gf = H.u16_to_f64(g)
    lr, _, _, eps, wd = hyper
    want = -lr * (gf / (np.abs(gf) + eps) + wd * theta0)
    got = H.u16_to_f64(deltas[0])
    # a dozen roundings of relative size 2^-9 each, applied to terms that may partly cancel
    tol = 12 * 2.0 ** -9 * lr * (np.abs(gf) / (np.abs(gf) + eps) + wd * np.abs(theta0)) + 1e-30
    assert np.all(np.abs(got - want) <= tol)
    # the alternative readings are far outside that tolerance for most elements
    inside_sqrt = -lr * (gf / np.sqrt(gf * gf + eps) + wd * theta0)
    no_bias_corr = -lr * (0.1 * gf / (np.sqrt(0.05) * np.abs(gf) + eps) + wd * theta0)
    assert np.mean(np.abs(got - inside_sqrt) > tol) > 0.9
    assert np.mean(np.abs(got - no_bias_corr) > tol) > 0.9
    # state after the step
    assert np.all(np.abs(H.u16_to_f64(st["m"]) - 0.1 * gf) <= 3 * 2.0 ** -9 * np.abs(0.1 * gf))
    vv = H.u16_to_f64(st["v"]) + (H.u16_to_f64(st["dv"]) if variant else 0.0)
    assert np.all(np.abs(vv - 0.05 * gf * gf) <= 4 * 2.0 ** -9 * 0.05 * gf * gf + 2.0 ** -133)
    new = H.u16_to_f64(st["theta"]) + H.u16_to_f64(st["dtheta"])
    pre = np.abs(theta0) >= np.abs(got)          # Grow's precondition |x| >= |a| (Alg. 1)
    assert pre.mean() > 0.95
    assert np.all(np.abs(new - (theta0 + got))[pre] <= 2.0 ** -15 * np.abs(theta0)[pre] + 2.0 ** -133)


@pytest.mark.parametrize("variant", [0, 1])
def test_first_step_closed_form_with_epsilon_under_the_root(orc, variant):
    """The flagged reading of line 12 as Alg. 2 prints it: delta = -lr * ( g / sqrt(g^2 + eps) + wd*theta ) at t = 1;
    the default reading (eps outside) is far outside the rounding tolerance, and nothing else changes."""
    n = 4096
    hyper = (1e-2, 0.9, 0.95, 4e-6, 0.5)          # eps comparable to g^2
    st = _state(n, 1, theta_std=1.0, plus=bool(variant))
    st_default = {k: (v.copy() if v is not None else None) for k, v in st.items()}
    theta0 = H.u16_to_f64(st["theta"])
    g = _grads(n, 1, 1, std=2e-3)
    deltas, deltas_default = [], []
    _run(orc, st, variant | orc.EPS_INSIDE_SQRT, hyper, 1, lambda t: g, deltas)
    _run(orc, st_default, variant, hyper, 1, lambda t: g, deltas_default)
    gf = H.u16_to_f64(g)
    lr, _, _, eps, wd = hyper
    want = -lr * (gf / np.sqrt(gf * gf + eps) + wd * theta0)
    got = H.u16_to_f64(deltas[0])
    tol = 12 * 2.0 ** -9 * lr * (np.abs(gf) / np.sqrt(gf * gf + eps) + wd * np.abs(theta0)) + 1e-30
    assert np.all(np.abs(got - want) <= tol)
    outside = -lr * (gf / (np.abs(gf) + eps) + wd * theta0)
    assert np.mean(np.abs(got - outside) > tol) > 0.9
    assert np.mean(deltas[0] != deltas_default[0]) > 0.9
    assert np.array_equal(st["m"], st_default["m"]) and np.array_equal(st["v"], st_default["v"])     # the moments do not see eps


# ------------------------------------------------------------------ tracks a textbook fp64 AdamW
@pytest.mark.parametrize("variant,beta2", [(0, 0.95), (1, 0.95), (1, 0.999)])
def test_tracks_fp64_adamw(orc, variant, beta2):
    n, steps = 20_000, 60
    hyper = (1e-3, 0.9, beta2, 1e-8, 0.1)
    st = _state(n, 2, theta_std=0.02, plus=bool(variant))
    theta0 = H.u16_to_f64(st["theta"])
    gs = [_grads(n, 2, t) for t in range(1, steps + 1)]
    _run(orc, st, variant, hyper, steps, lambda t: gs[t - 1])
    ref_theta, ref_m, ref_v = _torch_adamw_fp64(theta0, [H.u16_to_f64(g) for g in gs], hyper)
    got = H.u16_to_f64(st["theta"]) + H.u16_to_f64(st["dtheta"])
    moved = np.abs(ref_theta - theta0)
    assert np.median(moved) > 20 * 2.0 ** -9 * 0.02            # the run really moves the weights
    # m and v carry 8 significant bits, so each step's update is off by a few 2^-8 relative; errors of
    # 60 steps add up to well under 10% of the distance travelled plus one part in 2^14 of the weight
    err = np.abs(got - ref_theta)
    assert np.all(err <= 0.1 * steps * hyper[0] + 2.0 ** -14 * np.abs(theta0))
    assert np.median(err) <= 0.02 * np.median(moved)
    assert np.median(np.abs(H.u16_to_f64(st["m"]) - ref_m) / (np.abs(ref_m) + 1e-12)) < 2.0 ** -6
    vv = H.u16_to_f64(st["v"]) + (H.u16_to_f64(st["dv"]) if variant else 0.0)
    if not (variant == 0 and beta2 > 0.99):
        # the increment (1-beta2)*g^2 is one bf16 number in both variants (relative error up to 2^-8,
        # part of it the systematic rounding of 1-beta2); light adds the rounding of beta2 itself,
        # amplified by 1/(1-beta2), and of v at every step
        assert np.median(np.abs(vv - ref_v) / ref_v) < (2.0 ** -8 if variant else 2.0 ** -4)
    # plain bf16 accumulation of the same updates would not have moved at all for most elements:
    assert np.mean(np.abs(H.u16_to_f64(st["dtheta"])) > 0) > 0.9


def test_weight_decay_and_sign_are_in_the_update(orc):
    """Zero gradients: the only motion is the decay -lr*wd*theta per step (App. D), which plain bf16 loses."""
    n, steps = 2048, 200
    hyper = (1e-3, 0.9, 0.95, 1e-8, 0.1)
    st = _state(n, 3, theta_std=1.0)
    theta0 = H.u16_to_f64(st["theta"])
    zero = np.zeros(n, np.uint16)
    _run(orc, st, 0, hyper, steps, lambda t: zero)
    got = H.u16_to_f64(st["theta"]) + H.u16_to_f64(st["dtheta"])
    want = theta0 * (1 - hyper[0] * hyper[4]) ** steps
    # per step: B(wd), B(-lr) and two half-ulp roundings (< 1% of the step, partly systematic), plus Grow's
    # loss of at most half an ulp of the second component (2^-17 of theta)
    assert np.all(np.abs(got - want) <= 0.012 * np.abs(theta0 - want) + steps * 2.0 ** -17 * np.abs(theta0))
    assert np.all(np.abs(theta0 - want) > 0.015 * np.abs(theta0))
    assert np.all(np.abs(got) < np.abs(theta0))                 # decays towards zero: the sign is right
    assert np.all(st["m"] == 0) and np.all(st["v"] == 0)


def test_beta2_0p999_light_only_grows_plus_follows_average(orc):
    """Sec. 4.2: beta2 = 0.999 rounds to 1.0 in bf16, so the plain second moment never decreases;
    with (beta2, v) as expansions it follows the true moving average."""
    n = 4096
    hyper = (1e-4, 0.9, 0.999, 1e-8, 0.0)
    light, plus = _state(n, 4), _state(n, 4, plus=True)
    ema = np.zeros(n)
    prev = np.zeros(n)
    for t in range(1, 401):
        # gradient scale drops by 10x half way: a true average must come down again
        g = _grads(n, 4, t, std=1e-2 if t <= 200 else 1e-3)
        orc.adamw_step(light["theta"], light["dtheta"], light["m"], light["v"], None, g, 0, hyper, t)
        orc.adamw_step(plus["theta"], plus["dtheta"], plus["m"], plus["v"], plus["dv"], g, 1, hyper, t)
        gf = H.u16_to_f64(g)
        ema = 0.999 * ema + 0.001 * gf * gf
        lv = H.u16_to_f64(light["v"])
        assert np.all(lv >= prev)
        prev = lv
    pv = H.u16_to_f64(plus["v"]) + H.u16_to_f64(plus["dv"])
    rel_plus = np.abs(pv - ema) / ema
    rel_light = np.abs(prev - ema) / ema
    assert np.median(rel_plus) < 2.0 ** -9 and rel_plus.max() < 2.0 ** -6
    assert np.median(rel_light) > 0.05


def test_parameter_accumulation_identity(orc):
    """(theta_T + dtheta_T) equals theta_0 plus the fp64 sum of the bf16 updates the chain itself produced,
    up to the half-ulp-of-the-second-component loss per step; plain bf16 addition of the same updates stalls."""
    n, steps = 8192, 300
    hyper = (2.0 ** -16, 0.9, 0.95, 1e-8, 0.1)
    st = _state(n, 5, theta_std=1.0)
    theta0 = H.u16_to_f64(st["theta"])
    plain = st["theta"].copy()
    deltas = []
    _run(orc, st, 0, hyper, steps, lambda t: _grads(n, 5, t, mean=5e-4), deltas)
    total = theta0.copy()
    for d in deltas:
        total += H.u16_to_f64(d)
        plain = orc.binop(orc.ADD, plain, d)
    got = H.u16_to_f64(st["theta"]) + H.u16_to_f64(st["dtheta"])
    big = np.abs(theta0) > 0.05
    assert np.all(np.abs(got - total)[big] <= steps * 2.0 ** -17 * np.abs(theta0)[big])
    assert np.median(np.abs(got - total)[big] / np.abs(total - theta0)[big]) < 2.0 ** -6
    assert np.mean(plain[big] == H.np_round_f64_to_bf16(theta0)[big]) > 0.95      # lost arithmetic


def test_threads_do_not_change_results(orc):
    n = 10_007
    hyper = W.HYPER_PLUS_1P3B
    a, b = _state(n, 6, plus=True), _state(n, 6, plus=True)
    for t in range(1, 4):
        g = _grads(n, 6, t)
        orc.adamw_step(a["theta"], a["dtheta"], a["m"], a["v"], a["dv"], g, 1, hyper, t, nthreads=1)
        orc.adamw_step(b["theta"], b["dtheta"], b["m"], b["v"], b["dv"], g, 1, hyper, t, nthreads=7)
    for k in a:
        assert np.array_equal(a[k], b[k])


# ------------------------------------------------------------------ option D
def test_fp32_master_matches_fp64_adamw(orc):
    n, steps = 20_000, 50
    hyper = (1e-3, 0.9, 0.95, 1e-8, 0.1)
    theta = H.torch_to_u16(W.normal_bf16(n, 0.02, (7, 100)))
    master = H.u16_to_f32(theta).copy()
    m = np.zeros(n, np.float32)
    v = np.zeros(n, np.float32)
    gs = [_grads(n, 7, t) for t in range(1, steps + 1)]
    for t, g in enumerate(gs, 1):
        orc.fp32mw_step(theta, master, m, v, g, hyper, t)
    ref_theta, ref_m, ref_v = _torch_adamw_fp64(master * 0 + H.u16_to_f64(H.torch_to_u16(W.normal_bf16(n, 0.02, (7, 100)))),
                                               [H.u16_to_f64(g) for g in gs], hyper)
    assert np.max(np.abs(master - ref_theta) / (np.abs(ref_theta) + 1e-3)) < 2e-5
    assert np.max(np.abs(m - ref_m)) < 1e-6 * 1e-3            # fp32 rounding relative to the gradient scale
    assert np.max(np.abs(v - ref_v) / ref_v) < 1e-5
    assert np.array_equal(theta, orc.R_array(master))
