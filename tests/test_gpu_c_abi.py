"""The C ABI driven by a program written in plain C99 (paper_2405_03637_amd/csrc/abi_demo.c: HIP runtime
for memory, the library for everything else; no Python, no torch in that process).  The program writes its
final state to a file; here the same seeded inputs go through the oracle and the file must match bit for
bit, the fused EDQ of the last step within relative 1e-5."""
import os
import subprocess

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2405_03637_amd import build as lib_build

pytestmark = pytest.mark.gpu
M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix(x):
    with np.errstate(over="ignore"):
        x = x + np.uint64(0x9E3779B97F4A7C15)
        x = (x ^ (x >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        x = (x ^ (x >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return x ^ (x >> np.uint64(31))


def _pattern(seed, n, lo, span):
    """The generator of abi_demo.c: sign, exponent field in [lo, lo + span) and significand from one hash."""
    with np.errstate(over="ignore"):
        h = _mix(np.uint64(seed) * np.uint64(0x100000001B3) + np.arange(n, dtype=np.uint64))
    sign = (h >> np.uint64(63)).astype(np.uint32)
    expo = lo + ((h >> np.uint64(32)) % np.uint64(span)).astype(np.uint32)
    mant = (h & np.uint64(0x7F)).astype(np.uint32)
    return ((sign << 15) | (expo << 7) | mant).astype(np.uint16)


@pytest.mark.parametrize("variant", [orc.LIGHT, orc.PLUS, orc.LIGHT | orc.GROW_TWOSUM])
def test_plain_c_program_through_the_abi(variant, tmp_path):
    if not os.path.exists(lib_build.DEMO):
        lib_build.build_demo()
    n0, n1, steps = 70_001, 12_345, 4
    out = tmp_path / "state.bin"
    print(f"abi demo: variant {variant:#x}", flush=True)
    r = subprocess.run([lib_build.DEMO, str(out), str(variant), str(n0), str(n1), str(steps)],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    total = n0 + n1
    plus = (variant & 0xFF) == orc.PLUS
    theta = _pattern(1, total, 118, 10)
    z = lambda: np.zeros(total, np.uint16)
    dtheta, m, v, dv = z(), z(), z(), (z() if plus else None)
    hyper = (1e-3, 0.9, 0.95, 1e-8, 0.1)
    acc = orc.EdqAccumulator()
    for t in range(1, steps + 1):
        g = _pattern(100 + t, total, 110, 12)
        th0, dth0 = theta.copy(), dtheta.copy()
        d = np.empty(total, np.uint16)
        orc.adamw_step(theta, dtheta, m, v, dv, g, variant, hyper, t, delta_out=d)
        if t == steps:
            acc.add(d, th0, dth0, theta, dtheta)
    raw = np.fromfile(out, dtype=np.uint8)
    arrays = (5 if plus else 4)
    assert raw.size == arrays * total * 2 + 32
    got = raw[: arrays * total * 2].view(np.uint16).reshape(arrays, total)
    for k, (name, want) in enumerate((("theta", theta), ("dtheta", dtheta), ("m", m), ("v", v), ("dv", dv))[:arrays]):
        bad = np.flatnonzero(got[k] != want)
        assert bad.size == 0, f"{name}: {bad.size} mismatches, first at {int(bad[0])}"
    edq = raw[arrays * total * 2:].view(np.float64)
    assert abs(edq[0] - acc.value()) <= 1e-5 * abs(acc.value()) and int(edq[3]) == acc.lost.value
    assert np.count_nonzero(m) > 0.99 * total
