"""ctypes binding of the CPU oracle (mcf_oracle.cpp).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests/, the smoke check and the
benchmark's cpu_baseline leg may import this module.  The GPU library never
does, and this module never imports the GPU package.

bf16 arrays are numpy uint16 arrays (the upper half of an fp32 bit pattern); with fmt=FMT_FP16
the same uint16 arrays hold IEEE binary16 patterns and every step is done in that format.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mcf_oracle.cpp")
_LIB = os.path.join(_HERE, "libmcf_oracle.so")

ADD, SUB, MUL, DIV, SQRT = 0, 1, 2, 3, 4
LIGHT, PLUS, BF16, KAHAN, SGD = 0, 1, 2, 3, 4
GROW_TWOSUM = 0x100          # OR onto LIGHT or PLUS: Grow built on TwoSum
EPS_INSIDE_SQRT = 0x200      # OR onto any AdamW variant: epsilon under the root sign, as Alg. 2 prints line 12
FMT_BF16, FMT_FP16, FMT_E5M2, FMT_E4M3 = 0, 1, 2, 3    # component format ids (fmt= arguments)
STEP_FP16 = 0x1000           # OR onto the step's variant: fp16 arrays and scalars
STEP_E5M2, STEP_E4M3 = 0x2000, 0x3000      # FP8 arrays (one 8-bit pattern per uint16 element) and scalars


def step_flag(fmt):
    return fmt << 12


def build(force=False):
    """Compile the oracle with g++; one IEEE fp32 operation per written operation."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= max(
            os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "mcf_oracle.h"))):
        return _LIB
    cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
           "-pthread", "-o", _LIB, _SRC]
    subprocess.run(cmd, check=True)
    return _LIB


class Hyper(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("weight_decay", ctypes.c_double)]


class Scalars(ctypes.Structure):
    _fields_ = [(k, ctypes.c_uint16) for k in
                ("b1", "c1", "b2", "b2l", "c2", "bc1", "bc2", "e", "lam", "na")]


_u16p = ctypes.POINTER(ctypes.c_uint16)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    lib.orc_R.restype = ctypes.c_uint16
    lib.orc_R.argtypes = [ctypes.c_float]
    lib.orc_B.restype = ctypes.c_uint16
    lib.orc_B.argtypes = [ctypes.c_double]
    lib.orc_widen.restype = ctypes.c_float
    lib.orc_widen.argtypes = [ctypes.c_uint16]
    lib.orc_fp_env_ok.restype = ctypes.c_int
    lib.orc_R_array.argtypes = [_f32p, _u16p, ctypes.c_uint64]
    lib.orc_binop.argtypes = [ctypes.c_int, _u16p, _u16p, _u16p, ctypes.c_uint64]
    for name in ("orc_fast2sum", "orc_two_sum", "orc_two_prod_fma"):
        getattr(lib, name).argtypes = [_u16p, _u16p, _u16p, _u16p, ctypes.c_uint64]
    lib.orc_grow.argtypes = [_u16p, _u16p, _u16p, ctypes.c_uint64]
    lib.orc_grow_two_sum.argtypes = [_u16p, _u16p, _u16p, ctypes.c_uint64]
    lib.orc_mul_expansion.argtypes = [_u16p] * 6 + [ctypes.c_uint64]
    lib.orc_scaling.argtypes = [_u16p] * 5 + [ctypes.c_uint64]
    lib.orc_scalars_derive.argtypes = [ctypes.POINTER(Hyper), ctypes.c_uint64, ctypes.POINTER(Scalars)]
    lib.orc_adamw_step.argtypes = [_u16p] * 6 + [ctypes.c_uint64, ctypes.c_int, ctypes.POINTER(Hyper),
                                                ctypes.c_uint64, _u16p, ctypes.c_int]
    lib.orc_fp32mw_step.argtypes = [_u16p, _f32p, _f32p, _f32p, _u16p, ctypes.c_uint64,
                                    ctypes.POINTER(Hyper), ctypes.c_uint64, ctypes.c_int]
    lib.orc_edq_accumulate.argtypes = [_u16p] * 5 + [ctypes.c_uint64, _f64p, _f64p, ctypes.POINTER(ctypes.c_uint64)]
    lib.orc_R_fmt.restype = ctypes.c_uint16
    lib.orc_R_fmt.argtypes = [ctypes.c_int, ctypes.c_float]
    lib.orc_B_fmt.restype = ctypes.c_uint16
    lib.orc_B_fmt.argtypes = [ctypes.c_int, ctypes.c_double]
    lib.orc_widen_fmt.restype = ctypes.c_float
    lib.orc_widen_fmt.argtypes = [ctypes.c_int, ctypes.c_uint16]
    lib.orc_R_array_fmt.argtypes = [ctypes.c_int, _f32p, _u16p, ctypes.c_uint64]
    lib.orc_widen_array_fmt.argtypes = [ctypes.c_int, _u16p, _f32p, ctypes.c_uint64]
    lib.orc_binop_fmt.argtypes = [ctypes.c_int, ctypes.c_int, _u16p, _u16p, _u16p, ctypes.c_uint64]
    lib.orc_prim_fmt.argtypes = [ctypes.c_int, ctypes.c_int] + [_u16p] * 6 + [ctypes.c_uint64]
    lib.orc_scalars_derive_fmt.argtypes = [ctypes.c_int, ctypes.POINTER(Hyper), ctypes.c_uint64, ctypes.POINTER(Scalars)]
    lib.orc_edq_accumulate_fmt.argtypes = [ctypes.c_int] + [_u16p] * 5 + [ctypes.c_uint64, _f64p, _f64p,
                                                                          ctypes.POINTER(ctypes.c_uint64)]
    lib.orc_edq_finish.restype = ctypes.c_double
    lib.orc_edq_finish.argtypes = [ctypes.c_double, ctypes.c_double]
    lib.orc_set_array_threads.argtypes = [ctypes.c_int]
    lib.orc_set_array_threads(max(1, len(os.sched_getaffinity(0))))
    _lib = lib
    return lib


def _u16(a, writable=False):
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.dtype == np.uint16 and a.flags["C_CONTIGUOUS"], "need contiguous uint16"
    if writable:
        assert a.flags["WRITEABLE"]
    return a.ctypes.data_as(_u16p)


def _f32(a):
    assert isinstance(a, np.ndarray) and a.dtype == np.float32 and a.flags["C_CONTIGUOUS"] and a.flags["WRITEABLE"]
    return a.ctypes.data_as(_f32p)


def default_threads():
    return max(1, len(os.sched_getaffinity(0)))


# ---- scalar helpers -------------------------------------------------------
def R(f, fmt=FMT_BF16):
    """fp32 -> 16-bit pattern (RNE)."""
    return int(_load().orc_R_fmt(fmt, float(np.float32(f))))


def R_array(f, fmt=FMT_BF16):
    """fp32 array -> 16-bit patterns (RNE)."""
    f = np.ascontiguousarray(f, dtype=np.float32)
    out = np.empty(f.shape, np.uint16)
    _load().orc_R_array_fmt(fmt, f.ctypes.data_as(_f32p), _u16(out), f.size)
    return out


def B(x, fmt=FMT_BF16):
    """fp64 -> 16-bit pattern in one rounding."""
    return int(_load().orc_B_fmt(fmt, float(x)))


def widen(h, fmt=FMT_BF16):
    return float(_load().orc_widen_fmt(fmt, int(h)))


def widen_array(h, fmt=FMT_BF16):
    h = np.ascontiguousarray(h, dtype=np.uint16)
    out = np.empty(h.shape, np.float32)
    _load().orc_widen_array_fmt(fmt, _u16(h), out.ctypes.data_as(_f32p), h.size)
    return out


def fp_env_ok():
    return bool(_load().orc_fp_env_ok())


# ---- array operations -----------------------------------------------------
def binop(op, a, b=None, fmt=FMT_BF16):
    a = np.ascontiguousarray(a, dtype=np.uint16)
    if b is None:
        b = a
    b = np.ascontiguousarray(b, dtype=np.uint16)
    assert a.shape == b.shape
    out = np.empty_like(a)
    _load().orc_binop_fmt(fmt, op, _u16(a), _u16(b), _u16(out), a.size)
    return out


F2S, TWOSUM, GROW, GROW2, TWOPROD, SCALING, MULX = range(7)
_PRIM_INPUTS = {F2S: 2, TWOSUM: 2, GROW: 3, GROW2: 3, TWOPROD: 2, SCALING: 3, MULX: 4}


def prim(which, *inputs, fmt=FMT_BF16):
    """One of the seven expansion primitives over arrays; returns the two result arrays."""
    assert len(inputs) == _PRIM_INPUTS[which]
    arrs = [np.ascontiguousarray(t, dtype=np.uint16) for t in inputs]
    assert all(t.shape == arrs[0].shape for t in arrs)
    x = np.empty_like(arrs[0])
    y = np.empty_like(arrs[0])
    ptrs = [_u16(t) for t in arrs] + [None] * (4 - len(arrs))
    _load().orc_prim_fmt(fmt, which, *ptrs, _u16(x), _u16(y), x.size)
    return x, y


def fast2sum(a, b, fmt=FMT_BF16):
    return prim(F2S, a, b, fmt=fmt)


def two_sum(a, b, fmt=FMT_BF16):
    return prim(TWOSUM, a, b, fmt=fmt)


def two_prod_fma(a, b, fmt=FMT_BF16):
    return prim(TWOPROD, a, b, fmt=fmt)


def grow(x, y, a, fmt=FMT_BF16):
    """Returns new (x, y); inputs are not modified."""
    return prim(GROW, x, y, a, fmt=fmt)


def grow_two_sum(x, y, a, fmt=FMT_BF16):
    """Grow built on TwoSum.  Returns new (x, y); inputs are not modified."""
    return prim(GROW2, x, y, a, fmt=fmt)


def mul_expansion(a1, a2, b1, b2, fmt=FMT_BF16):
    return prim(MULX, a1, a2, b1, b2, fmt=fmt)


def scaling(v, a1, a2, fmt=FMT_BF16):
    return prim(SCALING, v, a1, a2, fmt=fmt)


def scalars(lr, beta1, beta2, eps, weight_decay, t, fmt=FMT_BF16):
    h = Hyper(lr, beta1, beta2, eps, weight_decay)
    s = Scalars()
    _load().orc_scalars_derive_fmt(fmt, ctypes.byref(h), int(t), ctypes.byref(s))
    return {k: getattr(s, k) for k, _ in Scalars._fields_}


def adamw_step(theta, dtheta, m, v, dv, grad, variant, hyper, t, delta_out=None, nthreads=None):
    """In-place Collage step over uint16 arrays.  hyper = (lr, beta1, beta2, eps, weight_decay).
    variant may carry GROW_TWOSUM and STEP_FP16."""
    n = theta.size
    base = variant & 0xFF
    for arr in (m, grad) + (() if base == BF16 else (dtheta,)) + (() if base == SGD else (v,)):
        assert arr.size == n
    if base == PLUS:
        assert dv is not None and dv.size == n
    if delta_out is not None:
        assert delta_out.size == n
    h = Hyper(*hyper)
    _load().orc_adamw_step(_u16(theta, True), None if base == BF16 else _u16(dtheta, True), _u16(m, True),
                           None if base == SGD else _u16(v, True), _u16(dv, True) if base == PLUS else None, _u16(grad), n, int(variant),
                           ctypes.byref(h), int(t), _u16(delta_out, True),
                           int(nthreads or default_threads()))


def fp32mw_step(theta, master, m, v, grad, hyper, t, nthreads=None):
    n = theta.size
    assert master.size == n and m.size == n and v.size == n and grad.size == n
    h = Hyper(*hyper)
    _load().orc_fp32mw_step(_u16(theta, True), _f32(master), _f32(m), _f32(v), _u16(grad), n,
                            ctypes.byref(h), int(t), int(nthreads or default_threads()))


class EdqAccumulator:
    """Sums the two EDQ totals over any number of slices, then finishes."""

    def __init__(self, fmt=FMT_BF16):
        self.fmt = fmt
        self.s1 = ctypes.c_double(0.0)
        self.s2 = ctypes.c_double(0.0)
        self.lost = ctypes.c_uint64(0)

    def add(self, delta, th0, dth0, th1, dth1):
        n = delta.size
        _load().orc_edq_accumulate_fmt(self.fmt, _u16(delta), _u16(th0), _u16(dth0), _u16(th1), _u16(dth1), n,
                                       ctypes.byref(self.s1), ctypes.byref(self.s2), ctypes.byref(self.lost))

    def value(self):
        return float(_load().orc_edq_finish(self.s1.value, self.s2.value))


def edq(delta, th0, dth0, th1, dth1, fmt=FMT_BF16):
    acc = EdqAccumulator(fmt)
    acc.add(delta, th0, dth0, th1, dth1)
    return acc.value()
