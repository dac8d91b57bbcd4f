"""Independent reference machinery for the tests.

Nothing here calls the oracle or the GPU library.  It provides
  * exact bf16 <-> rational conversions and a nearest-neighbour search over the
    table of all bf16 values (the definition of round-to-nearest-even), in pure
    Python with fractions.Fraction;
  * numpy conversions between bf16 bit patterns (uint16) and float64;
  * a vectorised float64 -> bf16 rounding in numpy, itself checked against the
    rational search in test_oracle_rounding.py.
"""
import bisect
from fractions import Fraction

import numpy as np

BF16_MAX_BITS = 0x7F7F           # largest finite
BF16_INF_BITS = 0x7F80


def bf16_bits_to_fraction(h):
    """Exact value of a finite bf16 bit pattern."""
    h = int(h)
    sign = -1 if h & 0x8000 else 1
    e = (h >> 7) & 0xFF
    mant = h & 0x7F
    assert e != 0xFF, "not finite"
    if e == 0:
        return sign * Fraction(mant, 1) * Fraction(1, 2 ** 133)       # subnormal: mant * 2^-126 * 2^-7
    return sign * Fraction(128 + mant, 1) * (Fraction(2) ** (e - 127 - 7))


# all non-negative finite bf16 values in increasing order; index == bit pattern
_POS = [bf16_bits_to_fraction(h) for h in range(0, BF16_MAX_BITS + 1)]
_OVERFLOW_MID = _POS[-1] + (_POS[-1] - _POS[-2]) / 2


def nearest_bf16(x):
    """Bit pattern of the bf16 nearest to the rational x, ties to even, IEEE overflow rule.
    The sign of a zero result follows the sign of x (x == 0 gives +0)."""
    x = Fraction(x)
    sign = 0x8000 if x < 0 else 0
    a = abs(x)
    if a >= _OVERFLOW_MID:
        return sign | BF16_INF_BITS
    i = bisect.bisect_right(_POS, a) - 1          # _POS[i] <= a
    lo = _POS[i]
    if lo == a or i == BF16_MAX_BITS:
        return sign | i
    hi = _POS[i + 1]
    dlo, dhi = a - lo, hi - a
    if dlo < dhi:
        return sign | i
    if dhi < dlo:
        return sign | (i + 1)
    return sign | (i if i % 2 == 0 else i + 1)    # tie: even mantissa == even bit pattern


def ulp_bf16(x):
    """Def. 3.1 with 7 stored mantissa bits: spacing at |x|."""
    a = abs(Fraction(x))
    if a == 0:
        return Fraction(1, 2 ** 133)
    e = 0
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    while Fraction(2) ** e > a:
        e -= 1
    return Fraction(2) ** (max(e, -126) - 7)


# ---- numpy side -------------------------------------------------------------
def u16_to_f64(u):
    u = np.asarray(u, dtype=np.uint16)
    return (u.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def u16_to_f32(u):
    u = np.asarray(u, dtype=np.uint16)
    return (u.astype(np.uint32) << 16).view(np.float32)


def f32_exact_to_u16(f):
    """fp32 values that are exactly representable in bf16 -> bits (asserts exactness)."""
    b = np.asarray(f, dtype=np.float32).view(np.uint32)
    assert np.all((b & 0xFFFF) == 0)
    return (b >> 16).astype(np.uint16)


def np_round_f64_to_bf16(x):
    """Vectorised float64 -> bf16 bits, one rounding, ties to even (finite or infinite x, no NaN).

    Works on the spacing: q = 2^(max(e,-126)-7); k = rint(|x|/q) (numpy rint is
    ties-to-even and |x|/q is exact); value k*q is then exactly representable in
    fp32, whose upper 16 bits are the answer."""
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    with np.errstate(divide="ignore", over="ignore", invalid="ignore"):
        _, e = np.frexp(a)
        e = e.astype(np.int64) - 1
        qe = np.maximum(e, -126) - 7
        k = np.rint(np.ldexp(a, (-qe).astype(np.int32)))
        val = np.ldexp(k, qe.astype(np.int32))
        val = np.where(np.isfinite(a), val, a)
        val = np.where(a == 0, 0.0, val)
        val = np.where(val >= float(_OVERFLOW_MID), np.inf, val)
        f = val.astype(np.float32)                  # exact (or inf)
    bits = f.view(np.uint32)
    assert np.all((bits & 0xFFFF) == 0)
    out = (bits >> 16).astype(np.uint16)
    return out | np.where(np.signbit(x), 0x8000, 0).astype(np.uint16)


def all_finite_bf16():
    """Every finite bf16 bit pattern, both signs."""
    pos = np.arange(0, BF16_MAX_BITS + 1, dtype=np.uint16)
    return np.concatenate([pos, pos | 0x8000])


def bf16_window(emin, emax, signs=True):
    """All bf16 patterns with unbiased exponent in [emin, emax] (normals), optionally both signs."""
    out = []
    for e in range(emin, emax + 1):
        base = (e + 127) << 7
        out.append(np.arange(base, base + 128, dtype=np.uint16))
    pos = np.concatenate(out)
    return np.concatenate([pos, pos | 0x8000]) if signs else pos


def torch_to_u16(t):
    """Bit patterns of a bf16/fp16 tensor, or of an FP8/uint8 tensor (one 8-bit pattern per uint16), as numpy uint16."""
    import torch
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16).copy()
    assert t.element_size() == 1
    return t.detach().cpu().contiguous().view(torch.uint8).numpy().astype(np.uint16)


def u16_to_torch(u, device="cpu", dtype=None):
    """16-bit patterns -> a torch tensor of dtype bfloat16 (default) or float16 holding those patterns."""
    import torch
    dtype = dtype or torch.bfloat16
    if dtype in (torch.bfloat16, torch.float16):
        return torch.from_numpy(np.ascontiguousarray(u).view(np.int16).copy()).view(dtype).to(device)
    return torch.from_numpy(np.ascontiguousarray(u).astype(np.uint8)).view(dtype).to(device)      # FP8: low byte of each pattern


def read_golden(path):
    rows = []
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [p.strip() for p in line.split("|")]
            rows.append(parts)
    return rows
