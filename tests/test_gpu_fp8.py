"""GPU parity for the two FP8 component formats (E5M2, E4M3): the HIP library against the CPU oracle,
bit for bit, through the C ABI.  Every stored 8-bit pattern identical; EDQ within relative 1e-5.
Single operations are checked over every operand pair, the rounding over all 2^32 fp32 patterns.
"""
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
FMTS = [2, 3]              # mcf_component and oracle format id: FP8 E5M2, FP8 E4M3
NAN = {2: 0x7E, 3: 0x7F}
ALL = np.arange(256, dtype=np.uint16)


def _dev(patterns):
    return torch.from_numpy(np.ascontiguousarray(patterns).astype(np.uint8)).to(DEV)


def _random_fp8(n, seed):
    """Half of the patterns uniform over all 256 (NaN, infinities, subnormals included), half in a narrow
    exponent band around 1 so that sums and differences really round."""
    rng = np.random.default_rng(seed)
    a = rng.integers(0, 256, n).astype(np.uint16)
    k = n // 2
    a[:k] = (rng.integers(0x30, 0x48, k) | (rng.integers(0, 2, k) << 7)).astype(np.uint16)
    return a


@pytest.mark.parametrize("fmt", FMTS)
def test_round_f32_to_fp8_all_patterns(fmt):
    """Every one of the 2^32 fp32 bit patterns through the library's rounding (the hardware conversion)
    against the oracle's R: round to nearest even, E5M2 overflow to infinity, E4M3 overflow to NaN."""
    chunk = 1 << 26
    out = torch.empty(chunk, dtype=torch.uint8, device=DEV)
    for c in range(0, 1 << 32, chunk):
        bits = torch.arange(c, c + chunk, dtype=torch.int64, device=DEV).to(torch.int32)
        mcf.round_f32_to(fmt, bits.view(torch.float32), out)
        got = H.torch_to_u16(out)
        want = orc.R_array(bits.cpu().numpy().view(np.float32), fmt=fmt)
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, f"fmt {fmt} chunk {c:#x}: {bad.size} mismatches, first at {c + int(bad[0]):#x}: " \
                              f"got {got[bad[0]]:#04x} want {want[bad[0]]:#04x}"
        if (c >> 26) % 16 == 15:
            _say(f"fp8 fmt {fmt} round: up to {c + chunk:#x} ok")


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("opname", ["add", "sub", "mul", "div", "sqrt"])
def test_fp8_op_every_pair(fmt, opname):
    op = {"add": 0, "sub": 1, "mul": 2, "div": 3, "sqrt": 4}[opname]
    if opname == "sqrt":
        a = _dev(ALL)
        out = torch.empty_like(a)
        mcf.component_op(fmt, op, a, None, out)
        got, want = H.torch_to_u16(out), orc.binop(op, ALL, fmt=fmt)
    else:
        aa, bb = np.repeat(ALL, 256), np.tile(ALL, 256)
        a_d, b_d = _dev(aa), _dev(bb)
        out = torch.empty_like(a_d)
        mcf.component_op(fmt, op, a_d, b_d, out)
        got, want = H.torch_to_u16(out), orc.binop(op, aa, bb, fmt=fmt)
    bad = np.flatnonzero(got != want)
    assert bad.size == 0, f"fmt {fmt} {opname}: {bad.size} mismatches, first operands {int(bad[0]) >> 8:#04x} {int(bad[0]) & 255:#04x} " \
                          f"got {got[bad[0]]:#04x} want {want[bad[0]]:#04x}"


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("n,shift", [(1, 0), (15, 1), (1000, 5), (262144 + 13, 7), (1 << 20, 0)])
def test_fp8_primitives(fmt, n, shift):
    """All seven expansion primitives on random bit patterns, buffers `shift` bytes past a 16-byte boundary."""
    arrs = [_random_fp8(n, 240 + k) for k in range(4)]
    pad = lambda u: _dev(np.concatenate([np.zeros(shift, np.uint16), u, np.zeros(16, np.uint16)]))
    full = [pad(u) for u in arrs]
    sl = slice(shift, shift + n)
    ins = [t[sl] for t in full]
    X, Y = torch.full_like(full[0], 7), torch.full_like(full[0], 7)
    guard = lambda t: (H.torch_to_u16(t[:shift]), H.torch_to_u16(t[shift + n:]))
    before = guard(X)
    cases = [(mcf.PRIM_FAST2SUM, orc.F2S, 2), (mcf.PRIM_TWOSUM, orc.TWOSUM, 2), (mcf.PRIM_GROW, orc.GROW, 3),
             (mcf.PRIM_GROW_TWOSUM, orc.GROW2, 3), (mcf.PRIM_TWOPROD, orc.TWOPROD, 2), (mcf.PRIM_SCALING, orc.SCALING, 3),
             (mcf.PRIM_MUL, orc.MULX, 4)]
    for code, ocode, nin in cases:
        mcf.primitive(fmt, code, ins[:nin], X[sl], Y[sl])
        wx, wy = orc.prim(ocode, *arrs[:nin], fmt=fmt)
        gx, gy = H.torch_to_u16(X[sl]), H.torch_to_u16(Y[sl])
        bad = np.flatnonzero((gx != wx) | (gy != wy))
        assert bad.size == 0, f"fmt {fmt} primitive {code}: {bad.size} mismatches, first at {int(bad[0])}: " \
                              f"inputs {[hex(int(u[bad[0]])) for u in arrs[:nin]]} got {gx[bad[0]]:#04x},{gy[bad[0]]:#04x} " \
                              f"want {wx[bad[0]]:#04x},{wy[bad[0]]:#04x}"
    assert all(np.array_equal(p, q) for p, q in zip(before, guard(X)))            # nothing outside was touched
    for u, t in zip(arrs, ins):
        assert np.array_equal(H.torch_to_u16(t), u)
    mcf.primitive(fmt, mcf.PRIM_GROW, ins[:3], ins[0], ins[1])                    # in place
    wx, wy = orc.grow(arrs[0], arrs[1], arrs[2], fmt=fmt)
    assert np.array_equal(H.torch_to_u16(ins[0]), wx) and np.array_equal(H.torch_to_u16(ins[1]), wy)


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("variant", ["light", "plus", "bf16", "kahan", "sgd", "light+twosum", "plus+twosum"])
def test_fp8_config1_flat_1m(fmt, variant):
    """One flat tensor of 2^20 FP8 parameters, 10 steps, every element after every step, fused EDQ; then the flat entry."""
    _say(f"fp8 fmt {fmt} config 1 {variant}")
    wl = Workload("flat_1m", variant=variant, fmt=fmt)
    full_oracle_run(wl, 10, edq=True)
    wl.close()
    wl = Workload("flat_1m", variant=variant, fmt=fmt)
    host = {k: H.torch_to_u16(getattr(wl, k)) for k in wl.state_names()}
    for t in range(1, 4):
        wl.new_grads(t)
        g = H.torch_to_u16(wl.grad)
        orc.adamw_step(host["theta"], host.get("dtheta"), host["m"], host.get("v"), host.get("dv"), g, wl.variant, wl.hyper, t)
        mcf.adamw_step_flat(wl.theta, wl.dtheta, wl.m, wl.v, wl.dv, wl.grad, wl.variant, wl.hyper, t)
    for k in wl.state_names():
        assert np.array_equal(H.torch_to_u16(getattr(wl, k)), host[k]), k
    wl.close()


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("variant", ["light", "plus", "sgd"])
def test_fp8_many_small_and_ragged_tensors(fmt, variant):
    """Tensors of 1..3000 one-byte elements back to back at odd byte offsets: heads, tails, the chunk table."""
    rng = np.random.default_rng(250)
    sizes = [int(x) for x in rng.integers(1, 3000, 200)] + [1, 2, 15, 16, 17, 31, 32, 33, 16383, 16384, 16385,
                                                            3 * 16384 + 5, 40_000, 100_003]
    shapes = [(f"t{i}", n) for i, n in enumerate(sizes)]
    for align in (1, 16):
        wl = Workload("flat_1m", variant=variant, shape_list=shapes, misalign_tiny=True, align=align, fmt=fmt)
        full_oracle_run(wl, 5, edq=True)
        wl.close()


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("variant", ["light", "plus", "bf16", "kahan", "sgd", "light+twosum", "plus+twosum"])
def test_fp8_special_values(fmt, variant):
    """State and gradients drawn from all bit patterns: NaN results come back as the one stored NaN,
    infinities (E5M2), overflow to NaN (E4M3), zeros and subnormals bit for bit."""
    n = 1 << 18
    wl = Workload("flat_1m", variant=variant, shape_list=[("a", n)], fmt=fmt)
    rnd = lambda s: _dev(_random_fp8(wl.total, s)).view(wl.dtype)
    wl.theta.copy_(rnd(260)); wl.m.copy_(rnd(262))
    if wl.v is not None:
        v = _random_fp8(wl.total, 263)
        v[: n // 2] &= 0x7F                       # mostly non-negative second moments keep a share of the elements finite
        wl.v.copy_(_dev(v).view(wl.dtype))
    if wl.dtheta is not None:
        wl.dtheta.copy_(rnd(261))
    if wl.dv is not None:
        wl.dv.copy_(rnd(264))
    host = {k: H.torch_to_u16(getattr(wl, k)) for k in wl.state_names()}
    for t in range(1, 4):
        wl.grad.copy_(rnd(270 + t))
        g = H.torch_to_u16(wl.grad)
        orc.adamw_step(host["theta"], host.get("dtheta"), host["m"], host.get("v"), host.get("dv"), g, wl.variant, wl.hyper, t)
        wl.plan.step(wl.hyper, t)
        for k in wl.state_names():
            dev = H.torch_to_u16(getattr(wl, k))
            bad = np.flatnonzero(dev != host[k])
            assert bad.size == 0, f"fmt {fmt} step {t} {k}: {bad.size} mismatches, first {int(bad[0])}: got {dev[bad[0]]:#04x} want {host[k][bad[0]]:#04x}"
    is_nan = (host["theta"] & 0x7F) > 0x7C if fmt == 2 else (host["theta"] & 0x7F) == 0x7F
    assert 0.005 < is_nan.mean() < 0.9999
    assert np.all(host["theta"][is_nan] == NAN[fmt])
    wl.close()


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("variant", ["light", "plus"])
def test_fp8_bias_corrections_of_many_steps_and_betas(fmt, variant):
    """The vector path multiplies by the fp16 reciprocal of each bias correction instead of dividing: one
    step from the same all-patterns state for many (beta1, beta2, t), so that the two corrections take
    most of the values they can, every element against the oracle.  The buffers start 3 bytes into their
    allocations, so the first and last slots go through the element path, which divides by the correction
    itself."""
    n = (1 << 16) - 7
    code = {"light": mcf.LIGHT, "plus": mcf.PLUS}[variant] | (fmt << 12)
    state0 = {k: _random_fp8(n, 300 + i) for i, k in enumerate(("theta", "dtheta", "m", "v", "dv", "grad"))}
    state0["v"] &= 0x7F
    if variant != "plus":
        state0["dv"] = None
    seen = set()
    tiny = 1.0 - 2.0 ** -16        # first-step correction 2^-16: E5M2's smallest number, whose reciprocal is no fp16 number
    for b1 in (0.0, 0.25, 0.5, 0.75, 0.875, tiny):
        for b2 in (0.5, 0.8125, 0.9375, 0.96875, tiny):
            hyper = (2.0 ** -6, b1, b2, 2.0 ** -6, 0.125)
            for t in (1, 2, 3, 4, 6, 9, 14, 40):
                bits = orc.scalars(*hyper, t, fmt=fmt)
                seen.add((int(bits["bc1"]), int(bits["bc2"])))
                host = {k: (None if v is None else v.copy()) for k, v in state0.items()}
                dev = {k: (None if v is None else _dev(np.concatenate([np.zeros(3, np.uint16), v]))[3:]) for k, v in state0.items()}
                orc.adamw_step(host["theta"], host["dtheta"], host["m"], host["v"], host["dv"], host["grad"], code, hyper, t)
                mcf.adamw_step_flat(dev["theta"], dev["dtheta"], dev["m"], dev["v"], dev["dv"], dev["grad"], code, hyper, t)
                for k in ("theta", "dtheta", "m", "v", "dv"):
                    if host[k] is None:
                        continue
                    got = H.torch_to_u16(dev[k])
                    bad = np.flatnonzero(got != host[k])
                    assert bad.size == 0, f"fmt {fmt} {variant} betas ({b1}, {b2}) step {t} {k}: {bad.size} mismatches, " \
                                          f"first {int(bad[0])}: got {got[bad[0]]:#04x} want {host[k][bad[0]]:#04x}"
        _say(f"fp8 fmt {fmt} {variant} beta1 {b1}: ok, {len(seen)} distinct correction pairs so far")
    assert len(seen) >= 12
    if fmt == 2:
        assert any(0x01 in pair for pair in seen)          # the corner was met


@pytest.mark.parametrize("fmt", FMTS)
def test_fp8_edq_standalone(fmt):
    n = 300_001
    rng = np.random.default_rng(280 + fmt)
    th0 = rng.integers(0x30, 0x48, n).astype(np.uint16) | (rng.integers(0, 2, n) << 7).astype(np.uint16)
    dth0 = rng.integers(0x00, 0x18, n).astype(np.uint16)
    delta = (rng.integers(0x08, 0x30, n) | (rng.integers(0, 2, n) << 7)).astype(np.uint16)
    th1, dth1 = orc.grow(th0, dth0, delta, fmt=fmt)
    scratch = torch.empty(mcf.edq_scratch_bytes(n), dtype=torch.uint8, device=DEV)
    out = torch.zeros(4, dtype=torch.float64, device=DEV)
    mcf.edq_component(fmt, _dev(delta), _dev(th0), _dev(dth0), _dev(th1), _dev(dth1), scratch, out)
    acc = orc.EdqAccumulator(fmt=fmt)
    acc.add(delta, th0, dth0, th1, dth1)
    got = out.cpu().numpy()
    assert abs(got[0] - acc.value()) <= 1e-5 * abs(acc.value()) and int(got[3]) == acc.lost.value
    plain = orc.binop(0, th0, delta, fmt=fmt)
    mcf.edq_component(fmt, _dev(delta), _dev(th0), None, _dev(plain), None, scratch, out)
    acc = orc.EdqAccumulator(fmt=fmt)
    acc.add(delta, th0, None, plain, None)
    got = out.cpu().numpy()
    assert abs(got[0] - acc.value()) <= 1e-5 * abs(acc.value()) and int(got[3]) == acc.lost.value > 0


@pytest.mark.parametrize("fmt", FMTS)
def test_fp8_llama_7b_sampled(fmt):
    """The 7B-shaped set with FP8 components (Collage-light, the launch configuration the benchmark times):
    three steps, sampled elements against the oracle."""
    _say(f"fp8 fmt {fmt} llama_7b: building")
    wl = Workload("llama_7b", fmt=fmt)
    idx = sample_indices(wl.shapes, wl.offs, seed=8)
    so = SampledOracle(wl, idx)
    edq_dev = torch.zeros(4, dtype=torch.float64, device=DEV)
    for t in range(1, 4):
        wl.new_grads(t)
        so.step(t)
        wl.plan.step(wl.hyper, t, edq_out=edq_dev if t == 3 else None)
        torch.cuda.synchronize()
        assert_bitwise(so.mismatches(), f"fp8 fmt {fmt} llama_7b step {t}")
        _say(f"fp8 fmt {fmt} llama_7b step {t}: {idx.size} sampled elements identical")
    assert edq_dev[0].item() > 0
    wl.close()
