"""GPU parity: the HIP library against the CPU oracle, bit for bit, through the C ABI.

Bar: every bf16 state element identical (integer comparison of the bit patterns); EDQ within
relative 1e-5 (fp64 reduction on both sides, different summation order).
"""
import os

import numpy as np
import pytest
import torch

import helpers as H
from conftest import say as _say
from gpu_harness import (SampledOracle, Workload, assert_bitwise, full_oracle_run, sample_indices, streamed_whole_state_check,
                         whole_state_run)
from oracle import oracle as orc
from paper_2405_03637_amd import binding as mcf
from paper_2405_03637_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _dev(u16):
    return H.u16_to_torch(u16, DEV)


# ------------------------------------------------------------------ rounding and single operations
def test_round_f32_all_patterns():
    """Every one of the 2^32 fp32 bit patterns through the library's rounding against the oracle's R."""
    chunk = 1 << 26
    out = torch.empty(chunk, dtype=torch.bfloat16, device=DEV)
    for c in range(0, 1 << 32, chunk):
        bits = torch.arange(c, c + chunk, dtype=torch.int64, device=DEV).to(torch.int32)   # wraps into the sign bit
        mcf.round_f32(bits.view(torch.float32), out)
        got = H.torch_to_u16(out)
        want = orc.R_array(bits.cpu().numpy().view(np.float32))
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, f"chunk {c:#x}: {bad.size} mismatches, first at {c + int(bad[0]):#x}"
    _say("round: 2^32 patterns ok")


@pytest.mark.parametrize("opname", ["add", "sub", "mul", "div", "sqrt"])
def test_bf16_op_sweep(opname):
    """The whole 2^16 x 2^16 operand table of every operation (MCF_QUICK_SWEEP=1: 1041 rows of it, except for
    div, whose fast route rests on a proof and is always swept in full); sqrt: all 2^16 inputs.
    Rows include zeros, subnormals, infinities and NaN patterns."""
    op = {"add": 0, "sub": 1, "mul": 2, "div": 3, "sqrt": 4}[opname]
    every = np.arange(1 << 16, dtype=np.uint16)
    if opname == "sqrt":
        a = _dev(every)
        out = torch.empty_like(a)
        mcf.bf16_op(op, a, None, out)
        assert np.array_equal(H.torch_to_u16(out), orc.binop(op, every))
        return
    if os.environ.get("MCF_QUICK_SWEEP") != "1" or opname == "div":
        rows = every
    else:
        rng = np.random.default_rng(30 + op)
        rows = np.unique(np.concatenate([rng.integers(0, 1 << 16, 1024).astype(np.uint16),
                                         np.array([0, 1, 0x7F, 0x80, 0x81, 0x3F80, 0x7F7F, 0x7F80, 0x7FC0, 0x8000, 0x8001,
                                                   0xBF80, 0xFF80, 0xFFFF, 0x0100, 0x7E80, 0x7F00], np.uint16)]))
    b = _dev(every)
    out = torch.empty_like(b)
    group = 64
    for i in range(0, rows.size, group):
        r = rows[i:i + group]
        aa = np.repeat(r, every.size)
        bb = np.tile(every, r.size)
        a_d, b_d = _dev(aa), _dev(bb)
        o_d = torch.empty_like(a_d)
        mcf.bf16_op(op, a_d, b_d, o_d)
        got = H.torch_to_u16(o_d)
        want = orc.binop(op, aa, bb)
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, f"{opname}: {bad.size} mismatches, first a={aa[bad[0]]:#06x} b={bb[bad[0]]:#06x} " \
                              f"got={got[bad[0]]:#06x} want={want[bad[0]]:#06x}"
        if (i // group) % 64 == 63:
            _say(f"bf16 {opname}: {i + group} rows ok")
    del out


def _random_bf16(n, seed, special=True):
    rng = np.random.default_rng(seed)
    a = rng.integers(0, 1 << 16, n).astype(np.uint16)
    k = n // 2
    # half of the values in a narrow exponent band so that sums and differences really round
    a[:k] = ((rng.integers(120, 134, k) << 7) | rng.integers(0, 128, k) | (rng.integers(0, 2, k) << 15)).astype(np.uint16)
    if not special:
        a[k:] = ((rng.integers(60, 190, n - k) << 7) | rng.integers(0, 128, n - k) | (rng.integers(0, 2, n - k) << 15)).astype(np.uint16)
    return a


@pytest.mark.parametrize("n,shift", [(1, 0), (7, 1), (64, 3), (1000, 5), (262144 + 13, 0), (262144 + 13, 7), (1 << 20, 0)])
def test_primitives(n, shift):
    """Fast2Sum, TwoSum and Grow on random bit patterns (NaN, infinities and subnormals included), with the
    buffers starting `shift` elements past a 16-byte boundary so that head and tail go element by element."""
    a, b, c = _random_bf16(n, 40), _random_bf16(n, 41), _random_bf16(n, 42)
    pad = lambda u: _dev(np.concatenate([np.zeros(shift, np.uint16), u, np.zeros(8, np.uint16)]))
    A, Bt, C = pad(a), pad(b), pad(c)
    X, Y = torch.full_like(A, 7.0), torch.full_like(A, 7.0)
    sl = slice(shift, shift + n)
    guard = lambda t: (H.torch_to_u16(t[:shift]), H.torch_to_u16(t[shift + n:]))
    before = guard(X)
    mcf.fast2sum(A[sl], Bt[sl], X[sl], Y[sl])
    wx, wy = orc.fast2sum(a, b)
    assert np.array_equal(H.torch_to_u16(X[sl]), wx) and np.array_equal(H.torch_to_u16(Y[sl]), wy)
    assert all(np.array_equal(p, q) for p, q in zip(before, guard(X)))            # nothing outside was touched
    mcf.two_sum(A[sl], Bt[sl], X[sl], Y[sl])
    wx, wy = orc.two_sum(a, b)
    assert np.array_equal(H.torch_to_u16(X[sl]), wx) and np.array_equal(H.torch_to_u16(Y[sl]), wy)
    mcf.grow(A[sl], Bt[sl], C[sl])
    wx, wy = orc.grow(a, b, c)
    assert np.array_equal(H.torch_to_u16(A[sl]), wx) and np.array_equal(H.torch_to_u16(Bt[sl]), wy)
    assert np.array_equal(H.torch_to_u16(C[sl]), c)


@pytest.mark.parametrize("n,shift", [(5, 1), (100_003, 0), (100_003, 3)])
def test_product_primitives_and_grow_on_two_sum(n, shift):
    """TwoProdFMA (Alg. 6), Scaling (Alg. 7), Mul (Alg. 8) and the TwoSum-based Grow on random bit patterns."""
    arrs = [_random_bf16(n, 45 + k) for k in range(4)]
    pad = lambda u: _dev(np.concatenate([np.zeros(shift, np.uint16), u, np.zeros(8, np.uint16)]))[shift:shift + n]
    A, Bt, C, D = (pad(u) for u in arrs)
    a, b, c, d = arrs
    X, Y = pad(np.zeros(n, np.uint16)), pad(np.zeros(n, np.uint16))
    mcf.two_prod_fma(A, Bt, X, Y)
    wx, wy = orc.two_prod_fma(a, b)
    assert np.array_equal(H.torch_to_u16(X), wx) and np.array_equal(H.torch_to_u16(Y), wy)
    mcf.scaling(A, Bt, C, X, Y)
    wx, wy = orc.scaling(a, b, c)
    assert np.array_equal(H.torch_to_u16(X), wx) and np.array_equal(H.torch_to_u16(Y), wy)
    mcf.mul(A, Bt, C, D, X, Y)
    wx, wy = orc.mul_expansion(a, b, c, d)
    assert np.array_equal(H.torch_to_u16(X), wx) and np.array_equal(H.torch_to_u16(Y), wy)
    mcf.grow_two_sum(A, Bt, C)
    wx, wy = orc.grow_two_sum(a, b, c)
    assert np.array_equal(H.torch_to_u16(A), wx) and np.array_equal(H.torch_to_u16(Bt), wy)


def test_primitives_mutually_misaligned_buffers():
    n = 5000
    a, b = _random_bf16(n, 43), _random_bf16(n, 44)
    A = _dev(np.concatenate([np.zeros(1, np.uint16), a]))[1:]
    Bt = _dev(np.concatenate([np.zeros(3, np.uint16), b]))[3:]
    X = torch.empty(n + 2, dtype=torch.bfloat16, device=DEV)[2:]
    Y = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    mcf.fast2sum(A, Bt, X, Y)
    wx, wy = orc.fast2sum(a, b)
    assert np.array_equal(H.torch_to_u16(X), wx) and np.array_equal(H.torch_to_u16(Y), wy)


# ------------------------------------------------------------------ the step: small, exhaustive comparisons
@pytest.mark.parametrize("variant", ["light", "plus", "bf16", "kahan", "sgd", "light+twosum", "plus+twosum"])
def test_config1_flat_1m(variant):
    """Config 1: one flat tensor of 2^20, 10 steps, every element after every step; plan and flat entry points."""
    _say(f"config 1 {variant}")
    wl = Workload("flat_1m", variant=variant)
    full_oracle_run(wl, 10, edq=True)
    wl.close()
    # the flat entry point on a fresh copy of the same inputs
    wl = Workload("flat_1m", variant=variant)
    host = {k: H.torch_to_u16(getattr(wl, k)) for k in wl.state_names()}
    for t in range(1, 4):
        wl.new_grads(t)
        g = H.torch_to_u16(wl.grad)
        orc.adamw_step(host["theta"], host.get("dtheta"), host["m"], host.get("v"), host.get("dv"), g, wl.variant, wl.hyper, t)
        mcf.adamw_step_flat(wl.theta, wl.dtheta, wl.m, wl.v, wl.dv, wl.grad, wl.variant, wl.hyper, t)
    for k in wl.state_names():
        assert np.array_equal(H.torch_to_u16(getattr(wl, k)), host[k]), k
    wl.close()


@pytest.mark.parametrize("variant", ["light", "plus", "bf16", "kahan", "sgd", "plus+twosum"])
def test_many_small_and_ragged_tensors(variant):
    """A few hundred tensors of 1..3000 elements packed back to back at odd offsets, plus three that span
    several chunks with ragged tails: exercises the chunk table, heads, tails and tiny tensors."""
    rng = np.random.default_rng(50)
    sizes = [int(x) for x in rng.integers(1, 3000, 300)] + [1, 2, 7, 8, 9, 15, 16, 17, 4095, 4096, 4097, 8191, 8193,
                                                            3 * 8192 + 5, 40_000, 100_003]
    shapes = [(f"t{i}", n) for i, n in enumerate(sizes)]
    for align in (1, 8):          # 1: every tensor starts wherever the previous one ended
        wl = Workload("flat_1m", variant=variant, shape_list=shapes, misalign_tiny=True, align=align,
                      hyper=W.HYPER_PLUS_1P3B if variant.startswith("plus") else W.HYPER_LIGHT)
        full_oracle_run(wl, 5, edq=True)
        wl.close()


@pytest.mark.parametrize("variant,fmt", [("light", 0), ("plus", 0), ("light", 1), ("plus", 2), ("light", 3)])
def test_buffers_at_different_offsets_modulo_16_bytes(variant, fmt):
    """Every stream of a tensor at its own offset from a 16-byte boundary (a gradient that is a view into a
    bucket, say): the slots are cut on theta's grid and the other streams are read and written with
    unaligned 128-bit accesses.  Two tensors, several chunks each; then the plan is pointed at gradients
    with yet another offset."""
    sizes = (200_003, 4_099)
    dtype = (torch.bfloat16, torch.float16, torch.float8_e5m2, torch.float8_e4m3fn)[fmt]
    code = {"light": mcf.LIGHT, "plus": mcf.PLUS}[variant] | (fmt << 12)
    hyper = W.HYPER_FP8 if fmt >= 2 else W.fp16_hyper(W.HYPER_LIGHT) if fmt == 1 else W.HYPER_LIGHT
    names = ["theta", "dtheta", "m", "v"] + (["dv"] if variant == "plus" else [])
    offsets = {"theta": 3, "dtheta": 0, "m": 5, "v": 2, "dv": 7, "grad": 1, "grad2": 6}
    dev, host = {}, {}
    for k in names + ["grad", "grad2"]:
        dev[k] = [torch.zeros(n + 16, dtype=torch.uint8 if fmt >= 2 else dtype, device=DEV).view(dtype)[offsets[k]:offsets[k] + n] for n in sizes]
    for i, n in enumerate(sizes):
        dev["theta"][i].copy_(W.normal_bf16(n, 0.02, (11, i), device=DEV).to(dtype))
    host = {k: [H.torch_to_u16(x) for x in dev[k]] for k in names}
    assert len({x.data_ptr() % 16 for k in names + ["grad"] for x in dev[k][:1]}) >= 4
    tensors = lambda g: [(dev["theta"][i], dev["dtheta"][i], dev["m"][i], dev["v"][i], dev["dv"][i] if variant == "plus" else None, dev[g][i])
                         for i in range(len(sizes))]
    plan = mcf.Plan(tensors("grad"), code)
    scale = W.FP16_LOSS_SCALE if fmt else 1.0
    for t in range(1, 5):
        gname = "grad" if t <= 2 else "grad2"
        if t == 3:
            plan.update(tensors("grad2"))
        for i, n in enumerate(sizes):
            dev[gname][i].copy_((W.normal_bf16(n, 1e-3, (11, 7, t, i), device=DEV).float() * scale).to(dtype))
            orc.adamw_step(host["theta"][i], host["dtheta"][i], host["m"][i], host["v"][i], host["dv"][i] if variant == "plus" else None,
                           H.torch_to_u16(dev[gname][i]), code, hyper, t)
        plan.step(hyper, t)
    torch.cuda.synchronize()
    for k in names:
        for i in range(len(sizes)):
            got = H.torch_to_u16(dev[k][i])
            bad = np.flatnonzero(got != host[k][i])
            assert bad.size == 0, f"{k}[{i}]: {bad.size} mismatches, first at {int(bad[0])}"
    plan.destroy()


@pytest.mark.parametrize("seed", range(int(os.environ.get("MCF_FUZZ_SEEDS", "48"))))      # 6648 seeds were run once: no mismatch
def test_seeded_mix_of_shapes_offsets_variants_and_formats(seed):
    """Plans drawn from a seed: 1 to 12 tensors of 1 to 60,000 elements (a few empty), every buffer of
    every tensor at its own element offset, any variant with any flag in any component format, one to
    three steps with the fused EDQ on the last.  Every element and the EDQ outputs against the oracle."""
    rng = np.random.default_rng(7000 + seed)
    fmt = int(rng.integers(0, 4))
    base = ["light", "plus", "bf16", "kahan", "sgd"][int(rng.integers(0, 5))]
    code = {"light": mcf.LIGHT, "plus": mcf.PLUS, "bf16": mcf.BF16, "kahan": mcf.KAHAN, "sgd": mcf.SGD}[base]
    if base in ("light", "plus") and rng.integers(0, 2):
        code |= mcf.GROW_TWOSUM
    if base != "sgd" and rng.integers(0, 4) == 0:
        code |= mcf.EPS_INSIDE_SQRT
    code |= fmt << 12
    dtype = (torch.bfloat16, torch.float16, torch.float8_e5m2, torch.float8_e4m3fn)[fmt]
    hyper = W.HYPER_FP8 if fmt >= 2 else W.fp16_hyper(W.HYPER_LIGHT) if fmt == 1 else W.HYPER_LIGHT
    names = ["theta"] + (["dtheta"] if base != "bf16" else []) + ["m"] + (["v"] if base != "sgd" else []) + (["dv"] if base == "plus" else [])
    sizes = [int(x) for x in rng.choice([0, 1, 7, 8, 9, 63, 64, 65, 511, 512, 513, 4097, 20_011, 60_000], int(rng.integers(1, 13)))]
    _say(f"seed {seed}: fmt {fmt} variant {code:#x} sizes {sizes}")
    aligned = bool(rng.integers(0, 2))               # half of the plans keep the buffers of a tensor mutually aligned
    dev = {k: [] for k in names + ["grad"]}
    for n in sizes:
        common = int(rng.integers(0, 16))
        for k in names + ["grad"]:
            off = common if aligned else int(rng.integers(0, 16))
            dev[k].append(torch.zeros(n + 32, dtype=torch.uint8 if fmt >= 2 else dtype, device=DEV).view(dtype)[off:off + n])
    for i, n in enumerate(sizes):
        if n:
            dev["theta"][i].copy_(W.normal_bf16(n, 0.02, (12, seed, i), device=DEV).to(dtype))
    host = {k: [H.torch_to_u16(x) for x in dev[k]] for k in names}
    get = lambda d, k, i: d[k][i] if k in d else None
    plan = mcf.Plan([(dev["theta"][i], get(dev, "dtheta", i), dev["m"][i], get(dev, "v", i), get(dev, "dv", i), dev["grad"][i])
                     for i in range(len(sizes))], code)
    assert plan.params == sum(sizes)
    steps = int(rng.integers(1, 4))
    scale = W.FP16_LOSS_SCALE if fmt else 1.0
    edq = torch.zeros(4, dtype=torch.float64, device=DEV)
    acc = orc.EdqAccumulator(fmt=fmt)
    for t in range(1, steps + 1):
        for i, n in enumerate(sizes):
            if not n:
                continue
            dev["grad"][i].copy_((W.normal_bf16(n, 1e-3, (12, seed, t, i), device=DEV).float() * scale).to(dtype))
            th0 = host["theta"][i].copy()
            dth0 = host["dtheta"][i].copy() if "dtheta" in host else None
            d = np.empty(n, np.uint16)
            orc.adamw_step(host["theta"][i], get(host, "dtheta", i), host["m"][i], get(host, "v", i), get(host, "dv", i),
                           H.torch_to_u16(dev["grad"][i]), code, hyper, t, delta_out=d)
            if t == steps:
                acc.add(d, th0, dth0, host["theta"][i], get(host, "dtheta", i))
        plan.step(hyper, t, edq_out=edq if t == steps else None)
    torch.cuda.synchronize()
    for k in names:
        for i in range(len(sizes)):
            got = H.torch_to_u16(dev[k][i])
            bad = np.flatnonzero(got != host[k][i])
            assert bad.size == 0, f"seed {seed} {k}[{i}] (n={sizes[i]}): {bad.size} mismatches, first at {int(bad[0])}"
    got = edq.cpu().numpy()
    assert abs(got[0] - acc.value()) <= 1e-5 * abs(acc.value()) + 1e-300 and int(got[3]) == acc.lost.value
    plan.destroy()


@pytest.mark.parametrize("variant", ["light", "plus", "bf16", "kahan", "sgd", "light+twosum", "plus+twosum"])
def test_special_values_take_the_exact_path(variant):
    """State and gradients drawn from all bit patterns (NaN, infinities, zeros, subnormals, huge and tiny
    values): the guarded fast arithmetic must hand these to the exact path and still match bit for bit."""
    n = 1 << 18
    shapes = [("a", n)]
    wl = Workload("flat_1m", variant=variant, shape_list=shapes)
    rnd = lambda s: _dev(_random_bf16(wl.total, s))
    wl.theta.copy_(rnd(60)); wl.m.copy_(rnd(62))
    if wl.v is not None:
        wl.v.copy_(rnd(63))
    if wl.dtheta is not None:
        wl.dtheta.copy_(rnd(61))
    if wl.dv is not None:
        wl.dv.copy_(rnd(64))
    # v must mostly be non-negative to keep a share of the elements finite
    if wl.v is not None:
        wl.v[: n // 2].abs_()
    host = {k: H.torch_to_u16(getattr(wl, k)) for k in wl.state_names()}
    for t in range(1, 4):
        wl.grad.copy_(rnd(70 + t))
        g = H.torch_to_u16(wl.grad)
        orc.adamw_step(host["theta"], host.get("dtheta"), host["m"], host.get("v"), host.get("dv"), g, wl.variant, wl.hyper, t)
        wl.plan.step(wl.hyper, t)
        for k in wl.state_names():
            dev = H.torch_to_u16(getattr(wl, k))
            bad = np.flatnonzero(dev != host[k])
            assert bad.size == 0, f"step {t} {k}: {bad.size} mismatches, first {int(bad[0])}: got {dev[bad[0]]:#06x} want {host[k][bad[0]]:#06x}"
    frac_nan = np.mean((host["theta"] & 0x7FFF) > 0x7F80)
    assert 0.005 < frac_nan < 0.9999
    wl.close()


def test_tiny_magnitudes_subnormal_intermediates():
    """Gradients around 1e-19..1e-22: v lands in and below the subnormal range, so quotients and roots meet
    subnormal intermediates; beta close to 1 and huge/zero eps are covered through the hyper-parameters."""
    n = 1 << 16
    for hyper in [(1e-3, 0.9, 0.95, 1e-8, 0.1), (1e-3, 0.9, 0.999, 0.0, 0.0), (1e-3, 0.0, 0.0, 1e-30, 0.01),
                  (1e-2, 0.99999, 0.9999999, 1e-8, 0.1)]:
        wl = Workload("flat_1m", variant="plus", shape_list=[("a", n)], hyper=hyper)
        host = {k: H.torch_to_u16(getattr(wl, k)) for k in wl.state_names()}
        rng = np.random.default_rng(80)
        for t in range(1, 5):
            scale = 10.0 ** rng.uniform(-24, -17, wl.total)
            gq = H.np_round_f64_to_bf16(rng.standard_normal(wl.total) * scale)
            gq[::97] = 0
            wl.grad.copy_(_dev(gq))
            orc.adamw_step(host["theta"], host["dtheta"], host["m"], host["v"], host["dv"], gq, 1, hyper, t)
            wl.plan.step(hyper, t)
            for k in wl.state_names():
                dev = H.torch_to_u16(getattr(wl, k))
                bad = np.flatnonzero(dev != host[k])
                assert bad.size == 0, f"hyper {hyper} step {t} {k}: {bad.size} mismatches"
        wl.close()


@pytest.mark.parametrize("variant", ["light", "plus", "kahan", "bf16", "light+twosum"])
def test_moments_decaying_into_the_subnormal_range(variant):
    """Parameters that stop receiving gradients: m and v shrink by beta every step, pass through the
    subnormal range and stick at the least subnormal numbers, so the bias-corrected moments, the root's
    operand and the quotient are subnormal step after step (the restricted arithmetic mode's second pass)."""
    n = 1 << 15
    hyper = (1e-3, 0.9, 0.95, 1e-8, 0.1)
    wl = Workload("flat_1m", variant=variant, shape_list=[("a", n - 5)], hyper=hyper)
    rng = np.random.default_rng(85)
    small = lambda lo, hi, signed: H.np_round_f64_to_bf16(2.0 ** rng.uniform(lo, hi, wl.total) *
                                                        (rng.choice([-1.0, 1.0], wl.total) if signed else 1.0))
    wl.m.copy_(_dev(small(-131, -118, True)))
    wl.v.copy_(_dev(small(-132, -116, False)))
    if wl.dv is not None:
        wl.dv.copy_(_dev(small(-133, -128, True)))
    host = {k: H.torch_to_u16(getattr(wl, k)) for k in wl.state_names()}
    zero = np.zeros(wl.total, np.uint16)
    wl.grad.zero_()
    for t in range(1, 61):
        orc.adamw_step(host["theta"], host.get("dtheta"), host["m"], host["v"], host.get("dv"), zero, wl.variant, hyper, t)
        wl.plan.step(hyper, t)
        if t in (1, 2, 5, 20, 60):
            for k in wl.state_names():
                dev = H.torch_to_u16(getattr(wl, k))[:n - 5]
                bad = np.flatnonzero(dev != host[k][:n - 5])
                assert bad.size == 0, f"{variant} step {t} {k}: {bad.size} mismatches, first at {int(bad[0])}"
    stuck = H.u16_to_f64(host["m"][:n - 5])
    # the first moments end up on the few least subnormal numbers that F(beta1 * m) maps to themselves
    assert float(np.mean((np.abs(stuck) > 0) & (np.abs(stuck) <= 2.0 ** -131))) > 0.5
    wl.close()


def test_checkpoint_resume_is_bitwise():
    """State is the tensors plus t: 6 steps equal 3 steps, a new plan, 3 more steps."""
    a = Workload("flat_1m", variant="plus", shape_list=[("x", 50_001), ("y", 333)], misalign_tiny=True)
    b = Workload("flat_1m", variant="plus", shape_list=[("x", 50_001), ("y", 333)], misalign_tiny=True)
    for t in range(1, 7):
        a.new_grads(t)
        b.grad.copy_(a.grad)
        a.plan.step(a.hyper, t)
        if t == 4:
            b.plan.destroy()
            tensors = [(b.theta[o:o + n], b.dtheta[o:o + n], b.m[o:o + n], b.v[o:o + n], b.dv[o:o + n], b.grad[o:o + n])
                       for (_, n), o in zip(b.shapes, b.offs)]
            b.plan = mcf.Plan(tensors, b.variant)
        b.plan.step(b.hyper, t)
    for k in a.state_names():
        assert torch.equal(getattr(a, k), getattr(b, k))
    a.close(); b.close()


def test_edq_standalone():
    n = 300_007
    rng = np.random.default_rng(90)
    th0 = H.np_round_f64_to_bf16(rng.standard_normal(n))
    delta = H.np_round_f64_to_bf16(rng.standard_normal(n) * 1e-3)
    dth0 = np.zeros(n, np.uint16)
    th1, dth1 = orc.grow(th0, dth0, delta)
    plain = orc.binop(orc.ADD, th0, delta)
    out = torch.zeros(4, dtype=torch.float64, device=DEV)
    scratch = torch.empty(mcf.edq_scratch_bytes(n) // 8, dtype=torch.float64, device=DEV)
    mcf.edq(_dev(delta), _dev(th0), _dev(dth0), _dev(th1), _dev(dth1), scratch, out)
    want = orc.edq(delta, th0, dth0, th1, dth1)
    assert abs(out[0].item() - want) <= 1e-5 * abs(want)
    mcf.edq(_dev(delta), _dev(th0), None, _dev(plain), None, scratch, out)      # Eq. 2 as printed: plain bf16
    want = orc.edq(delta, th0, None, plain, None)
    assert abs(out[0].item() - want) <= 1e-5 * abs(want)


EDGE_HYPERS = [
    # (lr, beta1, beta2, eps, weight_decay), step
    ((0.0, 0.9, 0.95, 1e-8, 0.1), 1),                    # no movement: delta = -0 * (...)
    ((1e-3, 0.0, 0.0, 0.0, 0.0), 1),                     # no memory, no epsilon: sign descent, 0/0 where g = 0
    ((1e-3, 0.9, 0.999, 1e-8, 0.0), 10 ** 9),            # bias corrections have reached 1
    ((1.0, 0.5, 0.5, 1.0, 1.0), 3),                      # everything of order one
    ((1e-3, 0.9, 0.95, 1e30, 0.1), 2),                   # epsilon dwarfs the root
    ((1e-3, 0.9, 0.95, 1e-40, 0.1), 2),                  # epsilon is a bf16 subnormal (0 in fp16)
    ((1e-3, 0.9, 1.0 - 1e-10, 1e-8, 0.1), 1),            # beta2 rounds to 1, 1-beta2 and its bias correction are tiny
    ((3e-4, 0.999999, 0.95, 1e-8, 0.1), 1),              # 1-beta1 = 1e-6
    ((1e4, 0.9, 0.95, 1e-8, 100.0), 5),                  # absurdly large step and decay: overflow to infinity and NaN
]


@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("variant", ["light", "plus", "sgd"])
def test_hyper_parameter_edge_cases(variant, fp16):
    """Extreme but valid hyper-parameters: whatever arithmetic mode the host picks for them, and whatever
    infinities and NaN they produce, every stored element must match the oracle."""
    shapes = [("a", 20_011), ("b", 3)]
    for hyper, t0 in EDGE_HYPERS:
        wl = Workload("flat_1m", variant=variant, shape_list=shapes, hyper=hyper, fp16=fp16, misalign_tiny=True)
        names = wl.state_names()
        host = {k: H.torch_to_u16(getattr(wl, k)) for k in names}
        live = np.zeros(wl.total, bool)                      # the oracle steps the arena's padding too; it is ignored
        for (_, n), o in zip(wl.shapes, wl.offs):
            live[o:o + n] = True
        for t in range(t0, t0 + 3):
            wl.new_grads(t)
            wl.grad[::5] = 0                                 # exact zeros among the gradients
            g = H.torch_to_u16(wl.grad)
            orc.adamw_step(host["theta"], host.get("dtheta"), host["m"], host.get("v"), host.get("dv"), g, wl.variant, hyper, t)
            wl.plan.step(hyper, t)
            for k in names:
                dev = H.torch_to_u16(getattr(wl, k))
                bad = np.flatnonzero((dev != host[k]) & live)
                assert not dev[~live].any()
                assert bad.size == 0, f"{variant} fp16={fp16} hyper {hyper} step {t} {k}: {bad.size} mismatches, first " \
                                      f"{int(bad[0])}: got {dev[bad[0]]:#06x} want {host[k][bad[0]]:#06x}"
        wl.close()


@pytest.mark.parametrize("fmt", [0, 1, 2, 3])
@pytest.mark.parametrize("variant", ["light", "plus", "bf16", "kahan", "plus+twosum"])
def test_epsilon_under_the_root_flag(variant, fmt):
    """MCF_EPS_INSIDE_SQRT (line 12 as Alg. 2 prints it) in every component format: ragged tensors, fused EDQ,
    plan and flat entry points; and it really is a different computation from the default."""
    shapes = [("a", 100_003), ("b", 5), ("c", 8192), ("d", 333)]
    eps = {0: 1e-6, 1: 1.0, 2: 2.0 ** -6, 3: 2.0 ** -6}[fmt]              # comparable to v_hat in that format's scaling
    base_h = W.HYPER_FP8 if fmt >= 2 else W.fp16_hyper(W.HYPER_LIGHT) if fmt == 1 else W.HYPER_LIGHT
    hyper = (base_h[0], base_h[1], base_h[2], eps, base_h[4])
    wl = Workload("flat_1m", variant=variant, shape_list=shapes, misalign_tiny=True, hyper=hyper, fmt=fmt)
    ref = Workload("flat_1m", variant=variant, shape_list=shapes, misalign_tiny=True, hyper=hyper, fmt=fmt)
    wl.plan.destroy()
    wl.variant |= mcf.EPS_INSIDE_SQRT                                       # the same bit in the oracle
    tensors = []
    for (_, n), o in zip(wl.shapes, wl.offs):
        sl = slice(o, o + n)
        tensors.append((wl.theta[sl], wl.dtheta[sl] if wl.dtheta is not None else None, wl.m[sl], wl.v[sl],
                        wl.dv[sl] if wl.dv is not None else None, wl.grad[sl]))
    wl.plan = mcf.Plan(tensors, wl.variant)
    full_oracle_run(wl, 4, edq=True)
    for t in range(1, 5):
        ref.new_grads(t)
        ref.plan.step(ref.hyper, t)
    torch.cuda.synchronize()
    assert not np.array_equal(H.torch_to_u16(wl.theta), H.torch_to_u16(ref.theta))       # the flag changes the trajectory
    assert np.array_equal(H.torch_to_u16(wl.m), H.torch_to_u16(ref.m))                    # but not the moments
    n = wl.shapes[0][1]
    flat = Workload("flat_1m", variant=variant, shape_list=[("a", n)], hyper=hyper, fmt=fmt)
    host = {k: H.torch_to_u16(getattr(flat, k)) for k in flat.state_names()}
    for t in range(1, 3):
        flat.new_grads(t)
        g = H.torch_to_u16(flat.grad)
        orc.adamw_step(host["theta"], host.get("dtheta"), host["m"], host.get("v"), host.get("dv"), g,
                       flat.variant | orc.EPS_INSIDE_SQRT, hyper, t)
        mcf.adamw_step_flat(flat.theta, flat.dtheta, flat.m, flat.v, flat.dv, flat.grad, flat.variant | mcf.EPS_INSIDE_SQRT, hyper, t)
    for k in flat.state_names():
        assert np.array_equal(H.torch_to_u16(getattr(flat, k))[:n], host[k][:n]), k
    for w in (wl, ref, flat):
        w.close()


def test_plan_update_repoints_the_plan():
    """mcf_plan_update: the same plan stepped over a second set of buffers (same sizes and alignment), then back;
    both trajectories follow the oracle; a set with another alignment is refused and leaves the plan usable."""
    shapes = [("a", 70_001), ("b", 5), ("c", 8192), ("d", 333)]
    a = Workload("flat_1m", variant="plus", shape_list=shapes, misalign_tiny=True, hyper=W.HYPER_PLUS_1P3B, seed=3)
    b = Workload("flat_1m", variant="plus", shape_list=shapes, misalign_tiny=True, hyper=W.HYPER_PLUS_1P3B, seed=4)
    def tensors(w, shift=0):
        return [(w.theta[o + shift:o + shift + n], w.dtheta[o + shift:o + shift + n], w.m[o + shift:o + shift + n],
                 w.v[o + shift:o + shift + n], w.dv[o + shift:o + shift + n], w.grad[o + shift:o + shift + n])
                for (_, n), o in zip(w.shapes, w.offs)]
    hosts = [{k: H.torch_to_u16(getattr(w, k)) for k in w.state_names()} for w in (a, b)]
    plan = a.plan
    t = 0
    for which in (0, 1, 0, 1):
        w, host = (a, b)[which], hosts[which]
        plan.update(tensors(w))
        for _ in range(2):
            t += 1
            w.new_grads(t)
            orc.adamw_step(host["theta"], host["dtheta"], host["m"], host["v"], host["dv"], H.torch_to_u16(w.grad), w.variant, w.hyper, t)
            plan.step(w.hyper, t)
        torch.cuda.synchronize()
        live = np.zeros(w.total, bool)
        for (_, n), o in zip(w.shapes, w.offs):
            live[o:o + n] = True
        for k in w.state_names():
            assert np.array_equal(H.torch_to_u16(getattr(w, k))[live], host[k][live]), (which, k)
    with pytest.raises(mcf.McfError) as e:                       # every tensor one element further: another alignment class
        plan.update([tuple(x[1:] for x in tt) for tt in tensors(b)][:1] + tensors(b)[1:])
    assert e.value.status in (mcf.MCF_ERR_SIZE, mcf.MCF_ERR_ALIGN)
    with pytest.raises(mcf.McfError):
        plan.update(tensors(b)[:-1])                             # a tensor short
    plan.update(tensors(a))                                      # still usable
    a.new_grads(99)
    orc.adamw_step(hosts[0]["theta"], hosts[0]["dtheta"], hosts[0]["m"], hosts[0]["v"], hosts[0]["dv"], H.torch_to_u16(a.grad), a.variant, a.hyper, 99)
    plan.step(a.hyper, 99)
    live = np.zeros(a.total, bool)
    for (_, n), o in zip(a.shapes, a.offs):
        live[o:o + n] = True
    assert np.array_equal(H.torch_to_u16(a.theta)[live], hosts[0]["theta"][live])
    a.close(); b.close()


def test_plan_update_in_bursts_without_synchronising():
    """mcf_plan_update is asynchronous: many updates and steps enqueued back to back, the gradients alternating
    between two buffers (as a framework that double-buffers them would), with no host synchronisation until the
    end.  Every step must have seen the table that was current when it was enqueued."""
    shapes = [("a", 200_003), ("b", 5), ("c", 8192)]
    wl = Workload("flat_1m", variant="light", shape_list=shapes, misalign_tiny=True)
    other = torch.zeros_like(wl.grad)
    grads = [wl.grad, other]
    def tensors(g):
        return [(wl.theta[o:o + n], wl.dtheta[o:o + n], wl.m[o:o + n], wl.v[o:o + n], None, g[o:o + n])
                for (_, n), o in zip(wl.shapes, wl.offs)]
    host = {k: H.torch_to_u16(getattr(wl, k)) for k in wl.state_names()}
    steps = 24
    host_grads = []
    for t in range(1, steps + 1):                     # draw every gradient first: nothing below waits for the device
        wl.new_grads(t)
        host_grads.append(H.torch_to_u16(wl.grad))
    dev_grads = [H.u16_to_torch(g, DEV) for g in host_grads]
    torch.cuda.synchronize()
    for t in range(1, steps + 1):
        g = grads[t & 1]
        g.copy_(dev_grads[t - 1], non_blocking=True)  # stream-ordered, like everything else here
        wl.plan.update(tensors(g))
        if t % 5 == 0:
            wl.plan.update(tensors(g))                # two updates in a row: the second reuses the first one's staging slot early
        wl.plan.step(wl.hyper, t)
    for t in range(1, steps + 1):
        orc.adamw_step(host["theta"], host["dtheta"], host["m"], host["v"], None, host_grads[t - 1], wl.variant, wl.hyper, t)
    torch.cuda.synchronize()
    for (_, n), o in zip(wl.shapes, wl.offs):
        for k in wl.state_names():
            assert np.array_equal(H.torch_to_u16(getattr(wl, k)[o:o + n]), host[k][o:o + n]), k
    wl.close()


def test_launch_pacing_changes_time_only():
    """mcf_set_launch_pacing: caps on the resident workgroups and idle time at either end of a wave move when the
    memory traffic happens, never what is computed.  A ragged set under several settings, every element against
    the oracle; the stream-mix measurement aid leaves the buffers it reads and rewrites in place as they were."""
    shapes = [("a", 300_007), ("b", 5), ("c", 8192), ("d", 333)]
    wl = Workload("flat_1m", variant="plus", shape_list=shapes, misalign_tiny=True, hyper=W.HYPER_PLUS_1P3B)
    try:
        settings = [(0, 0, 0), (1, 0, 0), (3, 7, 0), (12, 0, 9), (128, 33, 33), (-1, -1, -1)]
        host = {k: H.torch_to_u16(getattr(wl, k)) for k in wl.state_names()}
        for t, (groups, head, tail) in enumerate(settings, start=1):
            mcf.set_launch_pacing(groups, head, tail)
            wl.new_grads(t)
            orc.adamw_step(host["theta"], host["dtheta"], host["m"], host["v"], host["dv"], H.torch_to_u16(wl.grad), wl.variant, wl.hyper, t)
            wl.plan.step(wl.hyper, t)
            torch.cuda.synchronize()
            for (_, n), o in zip(wl.shapes, wl.offs):
                for k in wl.state_names():
                    assert np.array_equal(H.torch_to_u16(getattr(wl, k)[o:o + n]), host[k][o:o + n]), (groups, head, tail, k)
    finally:
        mcf.set_launch_pacing(-1, -1, -1)
    nb = wl.total // 8 * 8
    before = {k: getattr(wl, k).clone() for k in wl.state_names()}
    rd = [getattr(wl, k)[:nb] for k in ("theta", "dtheta", "m", "v", "dv", "grad")]
    for threads, vec, cap, store in ((64, 1, 10, 0), (256, 4, 0, 1), (64, 2, 3, 2)):
        mcf.stream_mix(rd, rd[:5], 2 * nb, threads, vec, cap, store)
        mcf.stream_mix(rd[:5], rd[:4], 2 * nb, threads, vec, cap, store)
    torch.cuda.synchronize()
    for k in wl.state_names():
        assert torch.equal(getattr(wl, k), before[k]), k
    dst = torch.zeros_like(wl.theta)
    mcf.stream_mix([wl.theta[:nb]], [dst[:nb]], 2 * nb, 256, 2, 0, 1)           # with distinct buffers it is a copy
    assert torch.equal(dst[:nb], wl.theta[:nb])
    wl.close()


def test_two_plans_on_two_streams():
    """Distinct plans are independent: two steps enqueued on two streams at once give the same bits as
    the oracle gives for each alone."""
    wls = [Workload("flat_1m", variant=v, shape_list=[("a", 3_000_017)], seed=s) for v, s in (("light", 1), ("plus", 2))]
    hosts = [{k: H.torch_to_u16(getattr(w, k)) for k in w.state_names()} for w in wls]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for t in range(1, 5):
        for w in wls:
            w.new_grads(t)
        torch.cuda.synchronize()
        for w, st in zip(wls, streams):
            w.plan.step(w.hyper, t, stream=st)
        for w, h in zip(wls, hosts):
            orc.adamw_step(h["theta"], h.get("dtheta"), h["m"], h.get("v"), h.get("dv"), H.torch_to_u16(w.grad), w.variant, w.hyper, t)
        torch.cuda.synchronize()
    for w, h in zip(wls, hosts):
        for k in w.state_names():
            n = w.shapes[0][1]                     # the oracle also stepped the arena's padding; compare the tensor
            assert np.array_equal(H.torch_to_u16(getattr(w, k))[:n], h[k][:n]), (w.variant, k)
        w.close()


# ------------------------------------------------------------------ option D
def test_fp32_master_baseline():
    shapes = [("a", 100_003), ("b", 77), ("c", 8192 * 3)]
    offs, total = W.layout(shapes)
    th = torch.zeros(total, dtype=torch.bfloat16, device=DEV)
    W.init_theta("flat_1m", shapes, offs, th)
    master = th.float()
    m = torch.zeros(total, dtype=torch.float32, device=DEV)
    v = torch.zeros_like(m)
    g = torch.zeros_like(th)
    plan = mcf.Fp32MwPlan([(th[o:o + n], master[o:o + n], m[o:o + n], v[o:o + n], g[o:o + n]) for (_, n), o in zip(shapes, offs)])
    h_th, h_w, h_m, h_v = H.torch_to_u16(th), master.cpu().numpy().copy(), m.cpu().numpy().copy(), v.cpu().numpy().copy()
    for t in range(1, 6):
        W.fill_grads("flat_1m", shapes, offs, g, t)
        orc.fp32mw_step(h_th, h_w, h_m, h_v, H.torch_to_u16(g), W.HYPER_LIGHT, t)
        plan.step(W.HYPER_LIGHT, t)
    live = np.zeros(total, bool)
    for (_, n), o in zip(shapes, offs):
        live[o:o + n] = True
    for name, host, dev in (("master", h_w, master), ("m", h_m, m), ("v", h_v, v)):
        d = dev.cpu().numpy()
        assert np.array_equal(d.view(np.uint32)[live], host.view(np.uint32)[live]), name
    assert np.array_equal(H.torch_to_u16(th)[live], h_th[live])
    plan.destroy()


def test_fp32_master_baseline_large_set():
    """The baseline over a set large enough (4 bytes x parameters >= 512 MiB) for the library to switch its stores to
    the write-through policy it uses on multi-gigabyte sets: two steps, every element of all four tensors."""
    shapes = [("big", (1 << 27) + 1003), ("b", 77), ("c", 12_345)]
    offs, total = W.layout(shapes)
    th = torch.zeros(total, dtype=torch.bfloat16, device=DEV)
    W.init_theta("flat_1m", shapes, offs, th)
    master = th.float()
    m = torch.zeros(total, dtype=torch.float32, device=DEV)
    v = torch.zeros_like(m)
    g = torch.zeros_like(th)
    plan = mcf.Fp32MwPlan([(th[o:o + n], master[o:o + n], m[o:o + n], v[o:o + n], g[o:o + n]) for (_, n), o in zip(shapes, offs)])
    h_th, h_w, h_m, h_v = H.torch_to_u16(th), master.cpu().numpy().copy(), m.cpu().numpy().copy(), v.cpu().numpy().copy()
    for t in (1, 2):
        W.fill_grads("flat_1m", shapes, offs, g, t)
        orc.fp32mw_step(h_th, h_w, h_m, h_v, H.torch_to_u16(g), W.HYPER_LIGHT, t)
        plan.step(W.HYPER_LIGHT, t)
        _say(f"fp32-master baseline, {total} elements: step {t} done")
    live = np.zeros(total, bool)
    for (_, n), o in zip(shapes, offs):
        live[o:o + n] = True
    for name, host, dev in (("master", h_w, master), ("m", h_m, m), ("v", h_v, v)):
        d = dev.cpu().numpy()
        assert np.array_equal(d.view(np.uint32)[live], host.view(np.uint32)[live]), name
    assert np.array_equal(H.torch_to_u16(th)[live], h_th[live])
    assert np.count_nonzero(h_m[live]) > 0.99 * live.sum()
    plan.destroy()


# ------------------------------------------------------------------ the paper-shaped configurations
def _sampled_steps(wl, so, first, last, check_at, on_grads=None):
    """Steps first..last of the library with the oracle following the sampled elements."""
    for t in range(first, last + 1):
        wl.new_grads(t)
        if on_grads is not None:
            on_grads(t)
        else:
            so.step(t)
        wl.plan.step(wl.hyper, t)
        if t in check_at:
            assert_bitwise(so.mismatches(), f"{wl.name} step {t}")
            _say(f"{wl.name}: step {t}: {so.idx.size} sampled elements identical")


def test_config2_gpt2_125m():
    """Config 2: 148 tensors, 124,439,808 parameters, light, 100 steps.  The oracle runs over every element for
    all 100 steps; every state tensor is compared whole at steps 1, 2, 10, 50 and 100."""
    wl = Workload("gpt2_125m")
    _say(f"gpt2_125m: {wl.n_params} params in {len(wl.shapes)} tensors")
    whole_state_run(wl, 100, {1, 2, 10, 50, 100}, _say)
    wl.close()


def test_config3_gpt_1p3b_plus_edq():
    """Config 3: 292 tensors, 1,315,819,520 parameters, plus, 20 steps, per-tensor gradient scales.  The oracle
    runs over every element for all 20 steps: the fused EDQ outputs (Def. 3.3; EDQ, both sums, lost count) are
    compared at every step, every state tensor whole at steps 1, 2, 5, 10 and 20."""
    wl = Workload("gpt_1p3b")
    _say(f"gpt_1p3b: {wl.n_params} params in {len(wl.shapes)} tensors")
    whole_state_run(wl, 20, {1, 2, 5, 10, 20}, _say, edq_every_step=True)
    wl.close()


def test_config4_llama_7b():
    """Config 4: 291 tensors, 6,738,415,616 parameters, light, 10 steps, in the launch configuration the
    benchmark times.  Steps 1 and 2: every element of every state tensor, streamed through the oracle piece by
    piece (the initial parameters, both gradient arenas and the state after step 1 stay on the device).  All 10
    steps: one seeded tensor of each large size (16.7 M, 45 M and 131 M elements) whole, and sampled elements of
    everything else (all small tensors, heads, tails and random windows of the large ones); the oracle follows
    both from step 0 on, compared at steps 1, 2, 5 and 10."""
    wl = Workload("llama_7b")
    names = wl.state_names()
    idx = sample_indices(wl.shapes, wl.offs)
    so = SampledOracle(wl, idx)
    by_size = {}
    for i, (_, n) in enumerate(wl.shapes):
        by_size.setdefault(n, []).append(i)
    rng = np.random.default_rng(4)
    chosen = [int(rng.choice(v)) for n, v in sorted(by_size.items()) if n > 16384]
    whole = {i: {k: H.torch_to_u16(getattr(wl, k)[wl.offs[i]:wl.offs[i] + wl.shapes[i][1]]) for k in names} for i in chosen}
    _say(f"llama_7b: {wl.n_params} params in {len(wl.shapes)} tensors, {idx.size} sampled, whole tensors "
         + ", ".join(f"{wl.shapes[i][0]} ({wl.shapes[i][1]})" for i in chosen))

    def follow(t):
        so.step(t)
        for i in chosen:
            o, n = wl.offs[i], wl.shapes[i][1]
            st = whole[i]
            orc.adamw_step(st["theta"], st["dtheta"], st["m"], st["v"], None, H.torch_to_u16(wl.grad[o:o + n]), wl.variant, wl.hyper, t)

    def check(t):
        assert_bitwise(so.mismatches(), f"llama_7b step {t}")
        for i in chosen:
            o, n = wl.offs[i], wl.shapes[i][1]
            for k in names:
                got = H.torch_to_u16(getattr(wl, k)[o:o + n])
                bad = np.flatnonzero(got != whole[i][k])
                assert bad.size == 0, f"llama_7b step {t} {wl.shapes[i][0]} {k}: {bad.size} of {n} differ, first at {int(bad[0])}"
        _say(f"llama_7b: step {t}: {idx.size} sampled elements and {len(chosen)} whole tensors identical")

    theta0 = wl.theta.clone()
    grads, snaps = [], []
    for t in (1, 2):
        wl.new_grads(t)
        follow(t)
        grads.append(wl.grad.clone() if t == 1 else wl.grad)
        wl.plan.step(wl.hyper, t)
        snaps.append({k: (getattr(wl, k).clone() if t == 1 else getattr(wl, k)) for k in names})
        check(t)
        if t == 1:
            # no chunk was skipped: after the first step m = F(c1 * g) is non-zero exactly where the gradient is (the
            # normal draws hold a few hundred exact zeros among 6.7e9; the arenas of this set have no padding)
            moved, drawn = int(torch.count_nonzero(wl.m).item()), int(torch.count_nonzero(wl.grad).item())
            assert moved == drawn and drawn > 0.999999 * wl.n_params, f"m is non-zero at {moved} elements, the gradient at {drawn} of {wl.n_params}"
    torch.cuda.synchronize()
    done = streamed_whole_state_check(wl, theta0, grads, snaps, _say)
    assert done == wl.n_params
    del theta0, grads, snaps
    torch.cuda.empty_cache()
    for t in range(3, 11):
        wl.new_grads(t)
        follow(t)
        wl.plan.step(wl.hyper, t)
        if t in (5, 10):
            check(t)
    wl.close()


@pytest.mark.parametrize("variant", ["plus", "kahan", "bf16", "sgd", "light+twosum", "plus+twosum"])
def test_llama_7b_other_strategies_sampled(variant):
    """The other strategies the benchmark times on the 7B-shaped set, in that launch configuration: three
    steps, sampled elements of every tensor against the oracle."""
    _say(f"llama_7b {variant}: building")
    wl = Workload("llama_7b", variant=variant)
    idx = sample_indices(wl.shapes, wl.offs, seed=9)
    so = SampledOracle(wl, idx)
    for t in range(1, 4):
        wl.new_grads(t)
        so.step(t)
        wl.plan.step(wl.hyper, t)
        torch.cuda.synchronize()
        assert_bitwise(so.mismatches(), f"llama_7b {variant} step {t}")
        _say(f"llama_7b {variant} step {t}: {idx.size} sampled elements identical")
    wl.close()


def test_config5_stress_64m():
    """Config 5: 64 Mi parameters incl. 4096 tensors of 1..256 elements at odd offsets, plus, lr = 2^-20,
    1000 steps.  Steps 1 to 100: the oracle over every element, whole state compared at steps 1, 10 and 100.  All
    1000 steps: every tiny tensor and windows of the large ones are followed by the oracle, compared at
    steps 10, 100, 500 and 1000, with the drift of theta + dtheta against the exact sum of the updates
    (Sec. 4: Grow keeps what a plain bf16 addition loses)."""
    name, steps = "stress_64m", 1000
    wl = Workload(name, misalign_tiny=True)
    idx = sample_indices(wl.shapes, wl.offs)
    so = SampledOracle(wl, idx)
    _say(f"{name}: {wl.n_params} params in {len(wl.shapes)} tensors, {idx.size} sampled")
    theta0 = H.u16_to_f64(so.state["theta"])
    track = {"ideal": theta0.copy(),                    # theta_0 + sum of the updates, in fp64
             "plain": so.state["theta"].copy()}         # the same updates added with plain bf16 addition (Eq. 1)

    def follow(t):
        delta = so.step(t, want_delta=True)
        track["ideal"] += H.u16_to_f64(delta)
        track["plain"] = orc.binop(orc.ADD, track["plain"], delta)

    whole_state_run(wl, 100, {1, 10, 100}, _say, on_grads=follow)
    assert_bitwise(so.mismatches(), f"{name} step 100")
    _sampled_steps(wl, so, 101, steps, {500, 1000}, on_grads=follow)
    # Drift of the DEVICE's expansion against the exact sum of the updates it was given.  Each Grow loses at
    # most half an ulp of the second component, i.e. at most 2^-16 of |theta| per step; plain bf16 never moves
    # because every update is below ulp/2.
    ideal, plain = track["ideal"], track["plain"]
    got = H.u16_to_f64(wl.gather(wl.theta, so.idx_dev)) + H.u16_to_f64(wl.gather(wl.dtheta, so.idx_dev))
    rel = np.abs(got - ideal) / np.abs(theta0)
    moved = np.abs(ideal - theta0) / np.abs(theta0)
    rel_plain = np.abs(H.u16_to_f64(plain) - ideal) / np.abs(theta0)
    _say(f"{name}: drift after {steps} steps: max {rel.max():.3e} rms {np.sqrt(np.mean(rel ** 2)):.3e} of |theta0|; "
         f"travelled median {np.median(moved):.3e}; plain bf16: max {rel_plain.max():.3e} rms "
         f"{np.sqrt(np.mean(rel_plain ** 2)):.3e}, unchanged {np.mean(plain == H.np_round_f64_to_bf16(theta0)):.3f}")
    assert rel.max() <= steps * 2.0 ** -16
    assert np.sqrt(np.mean(rel ** 2)) <= 8 * np.sqrt(steps) * 2.0 ** -17
    assert np.mean(plain == H.np_round_f64_to_bf16(theta0)) > 0.99          # lost arithmetic, Def. 3.2
    assert np.sqrt(np.mean(rel ** 2)) < 0.05 * np.sqrt(np.mean(rel_plain ** 2))
    wl.close()


def test_flat_tensor_longer_than_2_pow_32():
    """One flat tensor of 2^32 + 70,001 elements through the flat entry point and through a plan (64-bit
    element offsets in both): windows at the start, across the 2^31 and 2^32 boundaries and at the ragged end
    are followed by the oracle."""
    n = (1 << 32) + 70_001
    _say("flat > 2^32: allocating")
    z = lambda: torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    st = {"theta": z(), "dtheta": z(), "m": z(), "v": z()}
    grad = z()
    W.fill_grads("flat_1m", [("x", n)], [0], st["theta"], 0)          # any seeded bf16 values do
    st["theta"].mul_(20.0)
    w = 4096
    idx = np.unique(np.concatenate([np.arange(0, w), np.arange((1 << 31) - w, (1 << 31) + w),
                                    np.arange((1 << 32) - w, (1 << 32) + w), np.arange(n - w, n)]).astype(np.int64))
    idx_dev = torch.from_numpy(idx).to(DEV)
    host = {k: H.torch_to_u16(v[idx_dev]) for k, v in st.items()}
    plan = mcf.Plan([(st["theta"], st["dtheta"], st["m"], st["v"], None, grad)], mcf.LIGHT)     # 2^26 + 1095 chunks of one tensor
    for t in range(1, 5):
        W.fill_grads("flat_1m", [("x", n)], [0], grad, t)
        orc.adamw_step(host["theta"], host["dtheta"], host["m"], host["v"], None, H.torch_to_u16(grad[idx_dev]), 0,
                       W.HYPER_LIGHT, t)
        if t <= 2:
            mcf.adamw_step_flat(st["theta"], st["dtheta"], st["m"], st["v"], None, grad, mcf.LIGHT, W.HYPER_LIGHT, t)
        else:
            plan.step(W.HYPER_LIGHT, t)                 # the same tensor through the chunk table
    plan.destroy()
    for k, v in st.items():
        assert np.array_equal(H.torch_to_u16(v[idx_dev]), host[k]), k
    # and the step really ran everywhere: m is non-zero wherever the gradient is
    assert int(torch.count_nonzero(st["m"]).item()) > 0.99 * n


def test_step_replays_in_a_hip_graph():
    """The step allocates nothing and clears nothing with memsets, so it can be captured; every replay
    (with eager work and synchronisation in between) must reproduce the eager result bit for bit."""
    wl = Workload("flat_1m", variant="plus", shape_list=[("a", 300_001), ("b", 77), ("c", 4096)], misalign_tiny=True,
                  hyper=W.HYPER_PLUS_1P3B)
    wl.new_grads(1)
    snap = {k: getattr(wl, k).clone() for k in wl.state_names()}
    e_eager = torch.zeros(4, dtype=torch.float64, device=DEV)
    wl.plan.step(wl.hyper, 1, edq_out=e_eager)
    torch.cuda.synchronize()
    want = {k: getattr(wl, k).clone() for k in wl.state_names()}
    for k, v in snap.items():
        getattr(wl, k).copy_(v)
    e_graph = torch.zeros(4, dtype=torch.float64, device=DEV)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        wl.plan.step(wl.hyper, 1, edq_out=e_graph)
    for rep in range(3):
        for k, v in snap.items():
            getattr(wl, k).copy_(v)
        e_graph.zero_()
        _ = (wl.grad.float() * 2).sum().item()          # unrelated eager work and a synchronisation
        graph.replay()
        torch.cuda.synchronize()
        for k in wl.state_names():
            assert torch.equal(getattr(wl, k), want[k]), (rep, k)
        assert torch.equal(e_graph, e_eager), rep
    # mcf_plan_update refuses to be captured: its table copy would be replayed from whatever the staging memory holds later
    tensors = [(wl.theta[o:o + n], wl.dtheta[o:o + n], wl.m[o:o + n], wl.v[o:o + n], wl.dv[o:o + n], wl.grad[o:o + n])
               for (_, n), o in zip(wl.shapes, wl.offs)]
    scratch = torch.zeros(8, device=DEV)
    other = torch.cuda.CUDAGraph()
    with torch.cuda.graph(other):
        scratch.add_(1.0)                                # something to capture
        with pytest.raises(mcf.McfError) as err:
            wl.plan.update(tensors)
    assert err.value.status == mcf.MCF_ERR_HIP
    wl.plan.update(tensors)                              # outside a capture it is an ordinary call
    for k, v in snap.items():
        getattr(wl, k).copy_(v)
    wl.plan.step(wl.hyper, 1)
    torch.cuda.synchronize()
    for k in wl.state_names():
        assert torch.equal(getattr(wl, k), want[k]), k
    wl.close()


_EXACT_SCRIPT = r"""
import sys
sys.path.insert(0, sys.argv[1]); sys.path.insert(0, sys.argv[1] + "/tests")
import numpy as np, torch
import helpers as H
from gpu_harness import Workload
from oracle import oracle as orc
from paper_2405_03637_amd import workloads as W
for variant in ("light", "plus", "kahan", "bf16", "sgd", "plus+twosum"):
    shapes = [("a", 100_003), ("b", 5), ("c", 8192), ("d", 333)]
    wl = Workload("flat_1m", variant=variant, shape_list=shapes, misalign_tiny=True,
                  hyper=W.HYPER_PLUS_1P3B if variant.startswith("plus") else W.HYPER_LIGHT)
    host = {k: H.torch_to_u16(getattr(wl, k)) for k in wl.state_names()}
    edq = torch.zeros(4, dtype=torch.float64, device="cuda")
    for t in range(1, 4):
        wl.new_grads(t)
        orc.adamw_step(host["theta"], host.get("dtheta"), host["m"], host.get("v"), host.get("dv"),
                       H.torch_to_u16(wl.grad), wl.variant, wl.hyper, t)
        wl.plan.step(wl.hyper, t, edq_out=edq if t == 2 else None)
    torch.cuda.synchronize()
    for (_, n), o in zip(wl.shapes, wl.offs):
        for k in wl.state_names():
            assert np.array_equal(H.torch_to_u16(getattr(wl, k)[o:o + n]), host[k][o:o + n]), (variant, k)
    wl.close()
print("exact mode ok")
"""


def test_forced_exact_arithmetic_mode():
    """MCF_FORCE_EXACT=1 routes every step through the IEEE divide/sqrt, bit-pattern-rounding kernels (the
    ones the host falls back to for out-of-range hyper-parameters); they must match the oracle as well.
    The switch is read once per process, hence the child process."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ, MCF_FORCE_EXACT="1")
    r = subprocess.run([sys.executable, "-c", _EXACT_SCRIPT, root], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "exact mode ok" in r.stdout, r.stdout[-2000:] + r.stderr[-2000:]
