"""mcf_edq_noalloc, the stand-alone EDQ reduction (Def. 3.3) for callers that cannot allocate: its partials
live in a fixed array inside the library's device code instead of a caller's workspace.  Through the C ABI
it must give what mcf_edq_component gives with a workspace (same kernels, same summation order: the same
four doubles bit for bit) and agree with the oracle to relative 1e-5 with the lost count exact; two calls
in a row share the array, the second over a smaller input, and nothing is cleared in between."""
import numpy as np
import pytest
import torch

import helpers as H
from oracle import oracle as orc
from paper_2405_03637_amd import binding as mcf

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _inputs(n, seed, fmt):
    """delta, theta before, theta after one Grow, and a share of updates that a plain addition loses."""
    rng = np.random.default_rng(seed)
    if fmt == orc.FMT_BF16:
        th0 = H.np_round_f64_to_bf16(rng.standard_normal(n))
        delta = H.np_round_f64_to_bf16(rng.standard_normal(n) * 10.0 ** rng.uniform(-5, -2, n))
    else:
        th0 = orc.R_array((rng.standard_normal(n)).astype(np.float32), fmt=fmt)
        delta = orc.R_array((rng.standard_normal(n) * 10.0 ** rng.uniform(-5, -2, n)).astype(np.float32), fmt=fmt)
    dth0 = np.zeros(n, np.uint16)
    th1, dth1 = orc.grow(th0, dth0, delta, fmt=fmt)
    plain = orc.binop(orc.ADD, th0, delta, fmt=fmt)
    return delta, th0, dth0, th1, dth1, plain


@pytest.mark.parametrize("fmt", [orc.FMT_BF16, orc.FMT_FP16])
def test_noalloc_edq_matches_the_workspace_entry_point_and_the_oracle(fmt):
    dtype = torch.bfloat16 if fmt == orc.FMT_BF16 else torch.float16
    dev = lambda u: H.u16_to_torch(u, DEV, dtype)
    first = None
    for call, (n, shift) in enumerate([(3_000_017, 3), (70_001, 0), (5, 1)]):        # the later calls reuse a smaller part of the array
        print(f"noalloc edq: fmt {fmt} n {n} shift {shift}", flush=True)
        delta, th0, dth0, th1, dth1, plain = _inputs(n, 900 + call, fmt)
        pad = lambda u: dev(np.concatenate([np.zeros(shift, np.uint16), u]))[shift:]
        d_delta, d_th0, d_dth0, d_th1, d_dth1, d_plain = (pad(u) for u in (delta, th0, dth0, th1, dth1, plain))
        scratch = torch.empty(mcf.edq_scratch_bytes(n) // 8, dtype=torch.float64, device=DEV)
        for second0, second1, h0, h1, t1 in ((d_dth0, d_dth1, dth0, dth1, th1), (None, None, None, None, plain)):
            after = d_th1 if second1 is not None else d_plain
            with_ws = torch.full((4,), -1.0, dtype=torch.float64, device=DEV)
            without = torch.full((4,), -2.0, dtype=torch.float64, device=DEV)
            mcf.edq_component(fmt, d_delta, d_th0, second0, after, second1, scratch, with_ws)
            mcf.edq_noalloc(fmt, d_delta, d_th0, second0, after, second1, without)
            torch.cuda.synchronize()
            a, b = with_ws.cpu().numpy(), without.cpu().numpy()
            assert np.array_equal(a.view(np.uint64), b.view(np.uint64)), (n, a, b)
            acc = orc.EdqAccumulator(fmt=fmt)
            acc.add(delta, th0, h0, t1, h1)
            want = acc.value()
            assert abs(b[0] - want) <= 1e-5 * abs(want) + 1e-300, (n, b, want)
            assert abs(b[1] - acc.s1.value) <= 1e-5 * abs(acc.s1.value) + 1e-300
            assert abs(b[2] - acc.s2.value) <= 1e-5 * acc.s2.value
            assert int(b[3]) == acc.lost.value
            if second1 is None:
                assert acc.lost.value > 0                    # the plain addition really loses updates here
        if first is None:
            first = b.copy()
    # the first, largest input once more: what the smaller calls left in the array does not matter
    delta, th0, dth0, th1, dth1, plain = _inputs(3_000_017, 900, fmt)
    out = torch.zeros(4, dtype=torch.float64, device=DEV)
    pad = lambda u: dev(np.concatenate([np.zeros(3, np.uint16), u]))[3:]          # the first call's alignment, hence its summation order
    mcf.edq_noalloc(fmt, pad(delta), pad(th0), None, pad(plain), None, out)
    assert np.array_equal(out.cpu().numpy().view(np.uint64), first.view(np.uint64))


def test_noalloc_edq_limits_and_empty_input():
    out = torch.full((4,), 7.0, dtype=torch.float64, device=DEV)
    x = torch.zeros(8, dtype=torch.bfloat16, device=DEV)
    mcf.edq_noalloc(0, x, x, None, x, None, out, n=0)                 # an empty input writes zeros
    assert out.cpu().tolist() == [0.0, 0.0, 0.0, 0.0]
    with pytest.raises(mcf.McfError) as e:                            # beyond the fixed array: refused before any launch
        mcf.edq_noalloc(0, x, x, None, x, None, out, n=(1 << 28) + 1)
    assert e.value.status == mcf.MCF_ERR_SIZE
    with pytest.raises(mcf.McfError) as e:
        mcf.edq_noalloc(9, x, x, None, x, None, out)
    assert e.value.status == mcf.MCF_ERR_VARIANT
