"""Thin ctypes binding of libmcf_adamw.so: argument marshalling only.

Every step of the optimizer path runs in the library's HIP kernels; torch is used by callers
for device memory and streams.  Tensors are passed as torch tensors (bf16 or fp16, viewed through
their data_ptr) or as raw integer device addresses.  There is no CPU fallback: if the
library cannot be loaded, importing symbols from it raises.
"""
import ctypes
import os

from . import build as _build

_HERE = os.path.dirname(os.path.abspath(__file__))

MCF_OK = 0
MCF_ERR_NULL, MCF_ERR_SIZE, MCF_ERR_ALIGN, MCF_ERR_VARIANT, MCF_ERR_STEP, MCF_ERR_HYPER, MCF_ERR_HIP = \
    -1, -2, -3, -4, -5, -6, -7
LIGHT, PLUS, BF16, KAHAN, SGD = 0, 1, 2, 3, 4
GROW_TWOSUM = 0x100
EPS_INSIDE_SQRT = 0x200                        # OR onto any variant but SGD: epsilon under the root sign (Alg. 2 as printed)
FMT_FP16, FMT_FP8_E5M2, FMT_FP8_E4M3 = 0x1000, 0x2000, 0x3000      # OR onto a variant: tensors and scalars of that format
COMPONENT_BF16, COMPONENT_FP16, COMPONENT_FP8_E5M2, COMPONENT_FP8_E4M3 = 0, 1, 2, 3      # component format of the primitives
PRIM_FAST2SUM, PRIM_TWOSUM, PRIM_GROW, PRIM_GROW_TWOSUM, PRIM_TWOPROD, PRIM_SCALING, PRIM_MUL = range(7)
OP_ADD, OP_SUB, OP_MUL, OP_DIV, OP_SQRT = 0, 1, 2, 3, 4


class McfError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status} ({status_string(status)})")


class Hyper(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("weight_decay", ctypes.c_double)]


class Tensor(ctypes.Structure):
    _fields_ = [("theta", ctypes.c_void_p), ("dtheta", ctypes.c_void_p), ("m", ctypes.c_void_p),
                ("v", ctypes.c_void_p), ("dv", ctypes.c_void_p), ("grad", ctypes.c_void_p),
                ("n", ctypes.c_uint64)]


class Fp32Tensor(ctypes.Structure):
    _fields_ = [("theta", ctypes.c_void_p), ("master", ctypes.c_void_p), ("m", ctypes.c_void_p),
                ("v", ctypes.c_void_p), ("grad", ctypes.c_void_p), ("n", ctypes.c_uint64)]


_lib = None
_vp, _u64, _int = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int


def lib():
    """The loaded library.  Loads what is built; builds only if nothing is."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("MCF_LIBRARY") or _build.LIB        # MCF_LIBRARY: load another build of the library
    if not os.path.exists(path):
        _build.build()
    # torch owns the process's HIP runtime (device memory, streams): load it first so that this
    # library binds to the same libamdhip64 instead of bringing in a second copy
    import torch  # noqa: F401
    L = ctypes.CDLL(path)
    L.mcf_status_string.restype = ctypes.c_char_p
    L.mcf_status_string.argtypes = [_int]
    L.mcf_plan_create.argtypes = [ctypes.POINTER(_vp), ctypes.POINTER(Tensor), ctypes.c_uint32, _int]
    L.mcf_plan_destroy.argtypes = [_vp]
    L.mcf_plan_update.argtypes = [_vp, ctypes.POINTER(Tensor), ctypes.c_uint32, _vp]
    L.mcf_plan_params.restype = _u64
    L.mcf_plan_params.argtypes = [_vp]
    L.mcf_adamw_step.argtypes = [_vp, ctypes.POINTER(Hyper), _u64, _vp, _vp]
    L.mcf_step_scalars.argtypes = [_int, ctypes.POINTER(Hyper), _u64, ctypes.POINTER(ctypes.c_uint16), ctypes.POINTER(_int)]
    L.mcf_adamw_step_flat.argtypes = [_vp] * 6 + [_u64, _int, ctypes.POINTER(Hyper), _u64, _vp]
    L.mcf_fast2sum.argtypes = [_vp] * 4 + [_u64, _vp]
    L.mcf_two_sum.argtypes = [_vp] * 4 + [_u64, _vp]
    L.mcf_grow.argtypes = [_vp] * 3 + [_u64, _vp]
    L.mcf_grow_two_sum.argtypes = [_vp] * 3 + [_u64, _vp]
    L.mcf_two_prod_fma.argtypes = [_vp] * 4 + [_u64, _vp]
    L.mcf_scaling.argtypes = [_vp] * 5 + [_u64, _vp]
    L.mcf_mul.argtypes = [_vp] * 6 + [_u64, _vp]
    L.mcf_bf16_op.argtypes = [_int] + [_vp] * 3 + [_u64, _vp]
    L.mcf_round_f32.argtypes = [_vp, _vp, _u64, _vp]
    L.mcf_primitive.argtypes = [_int, _int] + [_vp] * 6 + [_u64, _vp]
    L.mcf_component_op.argtypes = [_int, _int] + [_vp] * 3 + [_u64, _vp]
    L.mcf_round_f32_to.argtypes = [_int, _vp, _vp, _u64, _vp]
    L.mcf_edq_component.argtypes = [_int] + [_vp] * 5 + [_u64, _vp, _vp, _vp]
    L.mcf_edq_noalloc.argtypes = [_int] + [_vp] * 5 + [_u64, _vp, _vp]
    L.mcf_edq_scratch_bytes.restype = _u64
    L.mcf_edq_scratch_bytes.argtypes = [_u64]
    L.mcf_edq.argtypes = [_vp] * 5 + [_u64, _vp, _vp, _vp]
    L.mcf_fp32mw_plan_create.argtypes = [ctypes.POINTER(_vp), ctypes.POINTER(Fp32Tensor), ctypes.c_uint32]
    L.mcf_fp32mw_plan_destroy.argtypes = [_vp]
    L.mcf_fp32mw_step.argtypes = [_vp, ctypes.POINTER(Hyper), _u64, _vp]
    L.mcf_stream_copy.argtypes = [_vp, _vp, _u64, _vp]
    L.mcf_set_launch_pacing.argtypes = [_int, _int, _int]
    L.mcf_stream_mix.argtypes = [ctypes.POINTER(_vp), ctypes.c_uint32, ctypes.POINTER(_vp), ctypes.c_uint32, _u64,
                                 ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32, _vp]
    _lib = L
    return L


def status_string(status):
    return lib().mcf_status_string(int(status)).decode()


def _check(status, where):
    if status != MCF_OK:
        raise McfError(status, where)


def _ptr(t):
    """Device address of a torch tensor, an int address, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("buffers must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _hyper(h):
    return h if isinstance(h, Hyper) else Hyper(*h)


class Plan:
    """mcf_plan over a list of (theta, dtheta, m, v, dv_or_None, grad) tensor tuples."""

    def __init__(self, tensors, variant):
        arr = (Tensor * max(1, len(tensors)))()
        self._keep = tensors
        for i, (th, dth, m, v, dv, g) in enumerate(tensors):
            n = th.numel() if hasattr(th, "numel") else None
            if n is None:
                raise TypeError("pass torch tensors; use Plan.raw for raw addresses")
            arr[i] = Tensor(_ptr(th), _ptr(dth), _ptr(m), _ptr(v), _ptr(dv), _ptr(g), n)
        self._h = _vp()
        _check(lib().mcf_plan_create(ctypes.byref(self._h), arr, len(tensors), int(variant)), "mcf_plan_create")
        self.variant = int(variant)

    @classmethod
    def raw(cls, entries, variant):
        """entries: list of (theta, dtheta, m, v, dv, grad, n) integer device addresses."""
        self = cls.__new__(cls)
        arr = (Tensor * max(1, len(entries)))()
        for i, e in enumerate(entries):
            arr[i] = Tensor(*e)
        self._keep = None
        self._h = _vp()
        _check(lib().mcf_plan_create(ctypes.byref(self._h), arr, len(entries), int(variant)), "mcf_plan_create")
        self.variant = int(variant)
        return self

    @property
    def params(self):
        return int(lib().mcf_plan_params(self._h))

    def update(self, tensors, stream=None):
        """Point the plan at other buffers of the same sizes and alignment (mcf_plan_update)."""
        arr = (Tensor * max(1, len(tensors)))()
        for i, (th, dth, m, v, dv, g) in enumerate(tensors):
            arr[i] = Tensor(_ptr(th), _ptr(dth), _ptr(m), _ptr(v), _ptr(dv), _ptr(g), th.numel())
        _check(lib().mcf_plan_update(self._h, arr, len(tensors), _stream(stream)), "mcf_plan_update")
        self._keep = tensors

    def step(self, hyper, t, stream=None, edq_out=None):
        """One optimizer step.  edq_out: optional float64 device tensor of 4 elements {EDQ, S1, S2, LOST}."""
        h = _hyper(hyper)
        _check(lib().mcf_adamw_step(self._h, ctypes.byref(h), int(t), _stream(stream), _ptr(edq_out)), "mcf_adamw_step")

    def destroy(self):
        if self._h:
            _check(lib().mcf_plan_destroy(self._h), "mcf_plan_destroy")
            self._h = _vp()
            self._keep = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class Fp32MwPlan:
    """mcf_fp32mw_plan over (theta_bf16, master_f32, m_f32, v_f32, grad_bf16) tuples."""

    def __init__(self, tensors):
        arr = (Fp32Tensor * max(1, len(tensors)))()
        self._keep = tensors
        for i, (th, w, m, v, g) in enumerate(tensors):
            arr[i] = Fp32Tensor(_ptr(th), _ptr(w), _ptr(m), _ptr(v), _ptr(g), th.numel())
        self._h = _vp()
        _check(lib().mcf_fp32mw_plan_create(ctypes.byref(self._h), arr, len(tensors)), "mcf_fp32mw_plan_create")

    def step(self, hyper, t, stream=None):
        h = _hyper(hyper)
        _check(lib().mcf_fp32mw_step(self._h, ctypes.byref(h), int(t), _stream(stream)), "mcf_fp32mw_step")

    def destroy(self):
        if self._h:
            _check(lib().mcf_fp32mw_plan_destroy(self._h), "mcf_fp32mw_plan_destroy")
            self._h = _vp()
            self._keep = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


SCALAR_NAMES = ("b1", "c1", "b2", "b2l", "c2", "bc1", "bc2", "e", "lam", "na")


def step_scalars(component, hyper, t):
    """The step's ten scalars as 16-bit patterns ({name: int}) and whether the reciprocal-based arithmetic applies."""
    h = _hyper(hyper)
    out = (ctypes.c_uint16 * 10)()
    ok = _int(0)
    _check(lib().mcf_step_scalars(int(component), ctypes.byref(h), int(t), out, ctypes.byref(ok)), "mcf_step_scalars")
    return dict(zip(SCALAR_NAMES, (int(x) for x in out))), bool(ok.value)


def adamw_step_flat(theta, dtheta, m, v, dv, grad, variant, hyper, t, stream=None, n=None):
    h = _hyper(hyper)
    n = theta.numel() if n is None else n
    _check(lib().mcf_adamw_step_flat(_ptr(theta), _ptr(dtheta), _ptr(m), _ptr(v), _ptr(dv), _ptr(grad), n,
                                     int(variant), ctypes.byref(h), int(t), _stream(stream)), "mcf_adamw_step_flat")


def fast2sum(a, b, x, y, stream=None):
    _check(lib().mcf_fast2sum(_ptr(a), _ptr(b), _ptr(x), _ptr(y), a.numel(), _stream(stream)), "mcf_fast2sum")


def two_sum(a, b, x, y, stream=None):
    _check(lib().mcf_two_sum(_ptr(a), _ptr(b), _ptr(x), _ptr(y), a.numel(), _stream(stream)), "mcf_two_sum")


def grow(x, y, a, stream=None):
    _check(lib().mcf_grow(_ptr(x), _ptr(y), _ptr(a), x.numel(), _stream(stream)), "mcf_grow")


def grow_two_sum(x, y, a, stream=None):
    _check(lib().mcf_grow_two_sum(_ptr(x), _ptr(y), _ptr(a), x.numel(), _stream(stream)), "mcf_grow_two_sum")


def two_prod_fma(a, b, x, e, stream=None):
    _check(lib().mcf_two_prod_fma(_ptr(a), _ptr(b), _ptr(x), _ptr(e), a.numel(), _stream(stream)), "mcf_two_prod_fma")


def scaling(v, a1, a2, x, e, stream=None):
    _check(lib().mcf_scaling(_ptr(v), _ptr(a1), _ptr(a2), _ptr(x), _ptr(e), v.numel(), _stream(stream)), "mcf_scaling")


def mul(a1, a2, b1, b2, x, e, stream=None):
    _check(lib().mcf_mul(_ptr(a1), _ptr(a2), _ptr(b1), _ptr(b2), _ptr(x), _ptr(e), a1.numel(), _stream(stream)), "mcf_mul")


def bf16_op(op, a, b, out, stream=None):
    _check(lib().mcf_bf16_op(int(op), _ptr(a), _ptr(b), _ptr(out), a.numel(), _stream(stream)), "mcf_bf16_op")


def round_f32(src, out, stream=None):
    _check(lib().mcf_round_f32(_ptr(src), _ptr(out), src.numel(), _stream(stream)), "mcf_round_f32")


def primitive(component, which, inputs, o0, o1, stream=None):
    """inputs: the 2 to 4 input tensors of the algorithm `which`; results go to (o0, o1)."""
    ps = [_ptr(t) for t in inputs] + [None] * (4 - len(inputs))
    _check(lib().mcf_primitive(int(component), int(which), *ps, _ptr(o0), _ptr(o1), inputs[0].numel(), _stream(stream)),
           "mcf_primitive")


def component_op(component, op, a, b, out, stream=None):
    _check(lib().mcf_component_op(int(component), int(op), _ptr(a), _ptr(b), _ptr(out), a.numel(), _stream(stream)),
           "mcf_component_op")


def round_f32_to(component, src, out, stream=None):
    _check(lib().mcf_round_f32_to(int(component), _ptr(src), _ptr(out), src.numel(), _stream(stream)), "mcf_round_f32_to")


def edq_component(component, delta, th0, dth0, th1, dth1, scratch, out, stream=None):
    _check(lib().mcf_edq_component(int(component), _ptr(delta), _ptr(th0), _ptr(dth0), _ptr(th1), _ptr(dth1), delta.numel(),
                                   _ptr(scratch), _stream(stream), _ptr(out)), "mcf_edq_component")


def edq_noalloc(component, delta, th0, dth0, th1, dth1, out, stream=None, n=None):
    _check(lib().mcf_edq_noalloc(int(component), _ptr(delta), _ptr(th0), _ptr(dth0), _ptr(th1), _ptr(dth1),
                                 delta.numel() if n is None else int(n), _stream(stream), _ptr(out)), "mcf_edq_noalloc")


def edq_scratch_bytes(n):
    return int(lib().mcf_edq_scratch_bytes(int(n)))


def edq(delta, th0, dth0, th1, dth1, scratch, out, stream=None):
    _check(lib().mcf_edq(_ptr(delta), _ptr(th0), _ptr(dth0), _ptr(th1), _ptr(dth1), delta.numel(),
                         _ptr(scratch), _stream(stream), _ptr(out)), "mcf_edq")


def stream_copy(dst, src, stream=None):
    nbytes = src.numel() * src.element_size()
    _check(lib().mcf_stream_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)), "mcf_stream_copy")


def set_launch_pacing(groups_per_cu=-1, head_sleep=-1, tail_sleep=-1):
    _check(lib().mcf_set_launch_pacing(int(groups_per_cu), int(head_sleep), int(tail_sleep)), "mcf_set_launch_pacing")


def stream_mix(reads, writes, nbytes, threads=64, vectors_per_lane=1, groups_per_cu=0, store_policy=0, stream=None):
    """reads, writes: lists of device tensors (or addresses); write j receives read j's data.
    store_policy: 0 non-temporal stores, 1 agent scope, 2 both."""
    r = (_vp * max(1, len(reads)))(*[_ptr(t) for t in reads])
    w = (_vp * max(1, len(writes)))(*[_ptr(t) for t in writes])
    _check(lib().mcf_stream_mix(r, len(reads), w, len(writes), int(nbytes), int(threads), int(vectors_per_lane),
                                int(groups_per_cu), int(store_policy), _stream(stream)), "mcf_stream_mix")


# ---- the C names, one to one (each returns nothing and raises McfError on a non-zero status) ----
def mcf_plan_create(tensors, variant):
    return Plan(tensors, variant)


def mcf_plan_destroy(plan):
    plan.destroy()


def mcf_plan_params(plan):
    return plan.params


def mcf_plan_update(plan, tensors, stream=None):
    plan.update(tensors, stream=stream)


def mcf_adamw_step(plan, hyper, step, stream=None, edq_dev=None):
    plan.step(hyper, step, stream=stream, edq_out=edq_dev)


mcf_adamw_step_flat = adamw_step_flat
mcf_step_scalars = step_scalars
mcf_fast2sum = fast2sum
mcf_two_sum = two_sum
mcf_grow = grow
mcf_grow_two_sum = grow_two_sum
mcf_two_prod_fma = two_prod_fma
mcf_scaling = scaling
mcf_mul = mul
mcf_bf16_op = bf16_op
mcf_round_f32 = round_f32
mcf_edq_scratch_bytes = edq_scratch_bytes
mcf_edq = edq
mcf_primitive = primitive
mcf_component_op = component_op
mcf_round_f32_to = round_f32_to
mcf_edq_component = edq_component
mcf_edq_noalloc = edq_noalloc
mcf_stream_copy = stream_copy
mcf_stream_mix = stream_mix
mcf_set_launch_pacing = set_launch_pacing
mcf_status_string = status_string


def mcf_fp32mw_plan_create(tensors):
    return Fp32MwPlan(tensors)


def mcf_fp32mw_plan_destroy(plan):
    plan.destroy()


def mcf_fp32mw_step(plan, hyper, step, stream=None):
    plan.step(hyper, step, stream=stream)
