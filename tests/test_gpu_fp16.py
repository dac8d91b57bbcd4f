"""GPU parity for the fp16 component format: the HIP library against the CPU oracle, bit for bit,
through the C ABI.  Same bar as for bf16: every stored 16-bit pattern identical; EDQ within relative 1e-5.
"""
import os

import numpy as np
import pytest
import torch

import helpers as H
from conftest import say as _say
from gpu_harness import SampledOracle, Workload, assert_bitwise, full_oracle_run, sample_indices
from oracle import oracle as orc
from paper_2405_03637_amd import binding as mcf
from paper_2405_03637_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"
F16 = orc.FMT_FP16
C16 = mcf.COMPONENT_FP16


def _dev(u16):
    return H.u16_to_torch(u16, DEV, torch.float16)


def _random_f16(n, seed):
    """Half of the patterns uniform over all 2^16 (NaN, infinities, subnormals included), half in a narrow
    exponent band so that sums and differences really round."""
    rng = np.random.default_rng(seed)
    a = rng.integers(0, 1 << 16, n).astype(np.uint16)
    k = n // 2
    a[:k] = ((rng.integers(10, 20, k) << 10) | rng.integers(0, 1024, k) | (rng.integers(0, 2, k) << 15)).astype(np.uint16)
    return a


def test_round_f32_to_fp16_all_patterns():
    """Every one of the 2^32 fp32 bit patterns through the library's fp16 rounding against the oracle's R."""
    chunk = 1 << 26
    out = torch.empty(chunk, dtype=torch.float16, device=DEV)
    for c in range(0, 1 << 32, chunk):
        bits = torch.arange(c, c + chunk, dtype=torch.int64, device=DEV).to(torch.int32)
        mcf.round_f32_to(C16, bits.view(torch.float32), out)
        got = H.torch_to_u16(out)
        want = orc.R_array(bits.cpu().numpy().view(np.float32), fmt=F16)
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, f"chunk {c:#x}: {bad.size} mismatches, first at {c + int(bad[0]):#x}"
        if (c >> 26) % 16 == 15:
            _say(f"fp16 round: up to {c + chunk:#x} ok")


@pytest.mark.parametrize("opname", ["add", "sub", "mul", "div", "sqrt"])
def test_fp16_op_sweep(opname):
    """The whole 2^16 x 2^16 operand table of every operation (MCF_QUICK_SWEEP=1: a thousand rows of it, except
    for div, always swept in full); sqrt: all 2^16 inputs."""
    op = {"add": 0, "sub": 1, "mul": 2, "div": 3, "sqrt": 4}[opname]
    every = np.arange(1 << 16, dtype=np.uint16)
    if opname == "sqrt":
        a = _dev(every)
        out = torch.empty_like(a)
        mcf.component_op(C16, op, a, None, out)
        assert np.array_equal(H.torch_to_u16(out), orc.binop(op, every, fmt=F16))
        return
    if os.environ.get("MCF_QUICK_SWEEP") != "1" or opname == "div":
        rows = every
    else:
        rng = np.random.default_rng(130 + op)
        rows = np.unique(np.concatenate([rng.integers(0, 1 << 16, 1024).astype(np.uint16),
                                         np.array([0, 1, 0x3FF, 0x400, 0x401, 0x3C00, 0x7BFF, 0x7C00, 0x7E00, 0x7C01, 0x8000,
                                                   0x8001, 0xBC00, 0xFC00, 0xFFFF, 0x0200, 0x7800], np.uint16)]))
    group = 64
    for i in range(0, rows.size, group):
        r = rows[i:i + group]
        aa = np.repeat(r, every.size)
        bb = np.tile(every, r.size)
        a_d, b_d = _dev(aa), _dev(bb)
        o_d = torch.empty_like(a_d)
        mcf.component_op(C16, op, a_d, b_d, o_d)
        got = H.torch_to_u16(o_d)
        want = orc.binop(op, aa, bb, fmt=F16)
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, f"{opname}: {bad.size} mismatches, first a={aa[bad[0]]:#06x} b={bb[bad[0]]:#06x} " \
                              f"got={got[bad[0]]:#06x} want={want[bad[0]]:#06x}"
        if (i // group) % 64 == 63:
            _say(f"fp16 {opname}: {i + group} rows ok")


@pytest.mark.parametrize("n,shift", [(1, 0), (7, 1), (1000, 5), (262144 + 13, 7), (1 << 20, 0)])
def test_fp16_primitives(n, shift):
    """All seven expansion primitives on random bit patterns, buffers `shift` elements past a 16-byte boundary."""
    arrs = [_random_f16(n, 140 + k) for k in range(4)]
    pad = lambda u: _dev(np.concatenate([np.zeros(shift, np.uint16), u, np.zeros(8, np.uint16)]))
    full = [pad(u) for u in arrs]
    sl = slice(shift, shift + n)
    ins = [t[sl] for t in full]
    X, Y = torch.full_like(full[0], 7.0), torch.full_like(full[0], 7.0)
    guard = lambda t: (H.torch_to_u16(t[:shift]), H.torch_to_u16(t[shift + n:]))
    before = guard(X)
    cases = [(mcf.PRIM_FAST2SUM, orc.F2S, 2), (mcf.PRIM_TWOSUM, orc.TWOSUM, 2), (mcf.PRIM_GROW, orc.GROW, 3),
             (mcf.PRIM_GROW_TWOSUM, orc.GROW2, 3), (mcf.PRIM_TWOPROD, orc.TWOPROD, 2), (mcf.PRIM_SCALING, orc.SCALING, 3),
             (mcf.PRIM_MUL, orc.MULX, 4)]
    for code, ocode, nin in cases:
        mcf.primitive(C16, code, ins[:nin], X[sl], Y[sl])
        wx, wy = orc.prim(ocode, *arrs[:nin], fmt=F16)
        gx, gy = H.torch_to_u16(X[sl]), H.torch_to_u16(Y[sl])
        bad = np.flatnonzero((gx != wx) | (gy != wy))
        assert bad.size == 0, f"primitive {code}: {bad.size} mismatches, first at {int(bad[0])}: " \
                              f"inputs {[hex(int(u[bad[0]])) for u in arrs[:nin]]} got {gx[bad[0]]:#06x},{gy[bad[0]]:#06x} " \
                              f"want {wx[bad[0]]:#06x},{wy[bad[0]]:#06x}"
    assert all(np.array_equal(p, q) for p, q in zip(before, guard(X)))            # nothing outside was touched
    for u, t in zip(arrs, ins):
        assert np.array_equal(H.torch_to_u16(t), u)                                # inputs untouched
    # Grow in place: results over the first two inputs
    mcf.primitive(C16, mcf.PRIM_GROW, ins[:3], ins[0], ins[1])
    wx, wy = orc.grow(arrs[0], arrs[1], arrs[2], fmt=F16)
    assert np.array_equal(H.torch_to_u16(ins[0]), wx) and np.array_equal(H.torch_to_u16(ins[1]), wy)


@pytest.mark.parametrize("variant", ["light", "plus", "bf16", "kahan", "sgd", "light+twosum", "plus+twosum"])
def test_fp16_config1_flat_1m(variant):
    """One flat tensor of 2^20 fp16 parameters, 10 steps, every element after every step, fused EDQ; then the flat entry."""
    _say(f"fp16 config 1 {variant}")
    wl = Workload("flat_1m", variant=variant, fp16=True)
    full_oracle_run(wl, 10, edq=True)
    wl.close()
    wl = Workload("flat_1m", variant=variant, fp16=True)
    host = {k: H.torch_to_u16(getattr(wl, k)) for k in wl.state_names()}
    for t in range(1, 4):
        wl.new_grads(t)
        g = H.torch_to_u16(wl.grad)
        orc.adamw_step(host["theta"], host.get("dtheta"), host["m"], host.get("v"), host.get("dv"), g, wl.variant, wl.hyper, t)
        mcf.adamw_step_flat(wl.theta, wl.dtheta, wl.m, wl.v, wl.dv, wl.grad, wl.variant, wl.hyper, t)
    for k in wl.state_names():
        assert np.array_equal(H.torch_to_u16(getattr(wl, k)), host[k]), k
    wl.close()


def test_fp16_unscaled_gradients_underflow_the_same_way():
    """Gradients of size 1e-3 with no loss scale: g^2 and v live among fp16's subnormals and flush to zero;
    whatever that does to the step, the library must do the same."""
    wl = Workload("flat_1m", variant="plus", fp16=True, hyper=W.HYPER_PLUS_1P3B)
    names = wl.state_names()
    host = {k: H.torch_to_u16(getattr(wl, k)) for k in names}
    for t in range(1, 5):
        W.fill_grads("flat_1m", wl.shapes, wl.offs, wl.grad, t)            # grad_scale 1
        g = H.torch_to_u16(wl.grad)
        orc.adamw_step(host["theta"], host["dtheta"], host["m"], host["v"], host["dv"], g, wl.variant, wl.hyper, t)
        wl.plan.step(wl.hyper, t)
        for k in names:
            dev = H.torch_to_u16(getattr(wl, k))
            bad = np.flatnonzero(dev != host[k])
            assert bad.size == 0, f"step {t} {k}: {bad.size} mismatches, first {int(bad[0])}: got {dev[bad[0]]:#06x} want {host[k][bad[0]]:#06x}"
    assert np.mean((host["v"] & 0x7C00) == 0) > 0.5          # most second moments are subnormal or zero
    wl.close()


@pytest.mark.parametrize("variant", ["light", "plus", "kahan", "sgd"])
def test_fp16_many_small_and_ragged_tensors(variant):
    rng = np.random.default_rng(150)
    sizes = [int(x) for x in rng.integers(1, 3000, 200)] + [1, 2, 7, 8, 9, 15, 16, 17, 4095, 4096, 4097, 8191, 8193,
                                                            3 * 8192 + 5, 40_000, 100_003]
    shapes = [(f"t{i}", n) for i, n in enumerate(sizes)]
    for align in (1, 8):
        wl = Workload("flat_1m", variant=variant, shape_list=shapes, misalign_tiny=True, align=align, fp16=True,
                      hyper=W.fp16_hyper(W.HYPER_PLUS_1P3B if variant.startswith("plus") else W.HYPER_LIGHT))
        full_oracle_run(wl, 5, edq=True)
        wl.close()


@pytest.mark.parametrize("variant", ["light", "plus", "bf16", "kahan", "sgd", "light+twosum", "plus+twosum"])
def test_fp16_special_values(variant):
    """State and gradients drawn from all bit patterns: NaN results must come back as the one stored NaN,
    infinities, zeros and subnormals bit for bit."""
    n = 1 << 18
    wl = Workload("flat_1m", variant=variant, shape_list=[("a", n)], fp16=True)
    rnd = lambda s: _dev(_random_f16(wl.total, s))
    wl.theta.copy_(rnd(160)); wl.m.copy_(rnd(162))
    if wl.v is not None:
        wl.v.copy_(rnd(163))
        wl.v[: n // 2].abs_()
    if wl.dtheta is not None:
        wl.dtheta.copy_(rnd(161))
    if wl.dv is not None:
        wl.dv.copy_(rnd(164))
    host = {k: H.torch_to_u16(getattr(wl, k)) for k in wl.state_names()}
    for t in range(1, 4):
        wl.grad.copy_(rnd(170 + t))
        g = H.torch_to_u16(wl.grad)
        orc.adamw_step(host["theta"], host.get("dtheta"), host["m"], host.get("v"), host.get("dv"), g, wl.variant, wl.hyper, t)
        wl.plan.step(wl.hyper, t)
        for k in wl.state_names():
            dev = H.torch_to_u16(getattr(wl, k))
            bad = np.flatnonzero(dev != host[k])
            assert bad.size == 0, f"step {t} {k}: {bad.size} mismatches, first {int(bad[0])}: got {dev[bad[0]]:#06x} want {host[k][bad[0]]:#06x}"
    frac_nan = np.mean((host["theta"] & 0x7FFF) > 0x7C00)
    assert 0.005 < frac_nan < 0.9999
    nan_bits = host["theta"][(host["theta"] & 0x7FFF) > 0x7C00]
    assert np.all(nan_bits == 0x7E00)
    wl.close()


def test_fp16_edq_standalone():
    n = 300_001
    th0, dth0 = _random_f16(n, 180), _random_f16(n, 181)
    keep = lambda u: np.where((u & 0x7C00) == 0x7C00, np.uint16(0x3C00), u)       # finite values only
    th0, dth0, delta = keep(th0), keep(dth0) & 0x83FF, keep(_random_f16(n, 182)) & 0x9FFF
    th1, dth1 = orc.grow(th0, dth0, delta, fmt=F16)
    scratch = torch.empty(mcf.edq_scratch_bytes(n), dtype=torch.uint8, device=DEV)
    out = torch.zeros(4, dtype=torch.float64, device=DEV)
    mcf.edq_component(C16, _dev(delta), _dev(th0), _dev(dth0), _dev(th1), _dev(dth1), scratch, out)
    acc = orc.EdqAccumulator(fmt=F16)
    acc.add(delta, th0, dth0, th1, dth1)
    got = out.cpu().numpy()
    assert abs(got[0] - acc.value()) <= 1e-5 * abs(acc.value())
    assert int(got[3]) == acc.lost.value
    mcf.edq_component(C16, _dev(delta), _dev(th0), None, _dev(th1), None, scratch, out)
    acc = orc.EdqAccumulator(fmt=F16)
    acc.add(delta, th0, None, th1, None)
    got = out.cpu().numpy()
    assert abs(got[0] - acc.value()) <= 1e-5 * abs(acc.value()) and int(got[3]) == acc.lost.value


def test_fp16_llama_7b_sampled():
    """The 7B-shaped set in fp16 (Collage-light, the launch configuration the benchmark times): three steps,
    sampled elements (heads, tails, unaligned windows, every small tensor) against the oracle."""
    _say("fp16 llama_7b: building")
    wl = Workload("llama_7b", fp16=True)
    idx = sample_indices(wl.shapes, wl.offs, seed=7)
    so = SampledOracle(wl, idx)
    edq_dev = torch.zeros(4, dtype=torch.float64, device=DEV)
    for t in range(1, 4):
        wl.new_grads(t)
        so.step(t)
        wl.plan.step(wl.hyper, t, edq_out=edq_dev if t == 3 else None)
        torch.cuda.synchronize()
        assert_bitwise(so.mismatches(), f"fp16 llama_7b step {t}")
        _say(f"fp16 llama_7b step {t}: {idx.size} sampled elements identical")
    got = edq_dev.cpu().numpy()
    assert got[0] > 0 and got[3] < wl.n_params // 100           # with the expansion almost no update is lost
    wl.close()
