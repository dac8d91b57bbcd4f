"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function
include/mcf.h declares, and reports argument errors before touching the device."""
import ctypes
import os
import re

import pytest
import torch

from paper_2405_03637_amd import binding as mcf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HAS_GPU = torch.cuda.is_available()


def _declared():
    text = open(os.path.join(ROOT, "include", "mcf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mcf_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = _declared()
    assert {"mcf_adamw_step", "mcf_adamw_step_flat", "mcf_plan_create", "mcf_plan_destroy", "mcf_grow", "mcf_fast2sum",
            "mcf_two_sum", "mcf_edq", "mcf_fp32mw_step", "mcf_bf16_op", "mcf_round_f32"} <= set(names)
    lib = mcf.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    for code in range(0, -8, -1):
        assert mcf.status_string(code) and mcf.status_string(code) != "unknown status"
    assert mcf.status_string(-99) == "unknown status"


def _hyper(**kw):
    d = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    d.update(kw)
    return mcf.Hyper(**d)


FAKE = 0x10000      # an aligned, non-NULL address that is never dereferenced on these paths


def _flat(theta=FAKE, dtheta=FAKE, m=FAKE, v=FAKE, dv=None, grad=FAKE, n=16, variant=0, hyper=None, step=1):
    h = hyper or _hyper()
    return mcf.lib().mcf_adamw_step_flat(theta, dtheta, m, v, dv, grad, n, variant, ctypes.byref(h), step, None)


def test_flat_step_argument_errors():
    assert _flat(theta=None) == mcf.MCF_ERR_NULL
    assert _flat(grad=None) == mcf.MCF_ERR_NULL
    assert _flat(variant=1, dv=None) == mcf.MCF_ERR_NULL
    assert _flat(variant=99) == mcf.MCF_ERR_VARIANT
    assert _flat(variant=mcf.SGD | mcf.GROW_TWOSUM) == mcf.MCF_ERR_VARIANT
    assert _flat(variant=mcf.BF16 | mcf.GROW_TWOSUM) == mcf.MCF_ERR_VARIANT     # the flag applies to Collage only
    assert _flat(variant=mcf.LIGHT | 0x400) == mcf.MCF_ERR_VARIANT
    assert _flat(variant=mcf.SGD | mcf.EPS_INSIDE_SQRT) == mcf.MCF_ERR_VARIANT         # SGD has no epsilon
    assert _flat(variant=mcf.PLUS | mcf.EPS_INSIDE_SQRT, dv=None) == mcf.MCF_ERR_NULL
    assert _flat(variant=mcf.LIGHT | 0x4000) == mcf.MCF_ERR_VARIANT
    assert _flat(variant=mcf.SGD | mcf.GROW_TWOSUM | mcf.FMT_FP8_E4M3) == mcf.MCF_ERR_VARIANT
    assert _flat(variant=mcf.LIGHT | mcf.FMT_FP8_E5M2, step=0) == mcf.MCF_ERR_STEP
    assert _flat(variant=mcf.LIGHT | mcf.FMT_FP8_E5M2, m=FAKE + 1, n=0) == mcf.MCF_OK
    assert _flat(variant=mcf.LIGHT | mcf.FMT_FP16, m=FAKE + 1) == mcf.MCF_ERR_ALIGN      # 2-byte elements need 2-byte alignment
    assert _flat(variant=mcf.SGD | mcf.GROW_TWOSUM | mcf.FMT_FP16) == mcf.MCF_ERR_VARIANT
    assert _flat(variant=mcf.PLUS | mcf.FMT_FP16, dv=None) == mcf.MCF_ERR_NULL       # the format flag changes no requirement
    assert _flat(variant=mcf.LIGHT | mcf.FMT_FP16, step=0) == mcf.MCF_ERR_STEP
    assert _flat(variant=3, dtheta=None) == mcf.MCF_ERR_NULL          # Kahan needs its variable
    assert _flat(variant=-1) == mcf.MCF_ERR_VARIANT
    assert _flat(m=FAKE + 1) == mcf.MCF_ERR_ALIGN
    assert _flat(n=(1 << 35) - 127) == mcf.MCF_ERR_SIZE
    assert _flat(step=0) == mcf.MCF_ERR_STEP
    assert _flat(hyper=_hyper(beta1=1.0)) == mcf.MCF_ERR_HYPER
    assert _flat(hyper=_hyper(beta2=-0.1)) == mcf.MCF_ERR_HYPER
    assert _flat(hyper=_hyper(lr=float("nan"))) == mcf.MCF_ERR_HYPER
    assert _flat(hyper=_hyper(eps=-1e-8)) == mcf.MCF_ERR_HYPER
    assert _flat(hyper=_hyper(weight_decay=float("inf"))) == mcf.MCF_ERR_HYPER
    assert mcf.lib().mcf_adamw_step_flat(FAKE, FAKE, FAKE, FAKE, None, FAKE, 16, 0, None, 1, None) == mcf.MCF_ERR_NULL
    # an empty tensor is a no-op and never reaches the device, whatever the pointers
    assert _flat(n=0, theta=None, grad=None) == mcf.MCF_OK


def test_plan_argument_errors():
    lib = mcf.lib()
    h = ctypes.c_void_p()
    one = (mcf.Tensor * 1)(mcf.Tensor(FAKE, FAKE, FAKE, FAKE, None, FAKE, 8))
    assert lib.mcf_plan_create(None, one, 1, 0) == mcf.MCF_ERR_NULL
    assert lib.mcf_plan_create(ctypes.byref(h), None, 1, 0) == mcf.MCF_ERR_NULL
    assert lib.mcf_plan_create(ctypes.byref(h), one, 1, 7) == mcf.MCF_ERR_VARIANT
    assert lib.mcf_plan_create(ctypes.byref(h), one, 1, 1) == mcf.MCF_ERR_NULL           # plus needs dv
    bad = (mcf.Tensor * 1)(mcf.Tensor(FAKE, FAKE + 1, FAKE, FAKE, None, FAKE, 8))
    assert lib.mcf_plan_create(ctypes.byref(h), bad, 1, 0) == mcf.MCF_ERR_ALIGN
    big = (mcf.Tensor * 1)(mcf.Tensor(FAKE, FAKE, FAKE, FAKE, None, FAKE, (1 << 35) - 127))
    assert lib.mcf_plan_create(ctypes.byref(h), big, 1, 0) == mcf.MCF_ERR_SIZE
    assert not h.value
    hy = _hyper()
    assert lib.mcf_adamw_step(None, ctypes.byref(hy), 1, None, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_plan_destroy(None) == mcf.MCF_OK
    assert lib.mcf_plan_params(None) == 0
    # a plan over nothing needs no device memory and its step does nothing
    assert lib.mcf_plan_create(ctypes.byref(h), None, 0, 0) == mcf.MCF_OK and h.value
    assert lib.mcf_adamw_step(h, ctypes.byref(hy), 0, None, None) == mcf.MCF_ERR_STEP
    assert lib.mcf_adamw_step(h, None, 1, None, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_adamw_step(h, ctypes.byref(hy), 1, None, FAKE + 4) == mcf.MCF_ERR_ALIGN
    assert lib.mcf_adamw_step(h, ctypes.byref(hy), 1, None, None) == mcf.MCF_OK
    assert lib.mcf_plan_destroy(h) == mcf.MCF_OK
    # mcf_plan_update: argument errors come before any device work (a plan over nothing has no table to copy)
    assert lib.mcf_plan_update(None, one, 1, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_plan_create(ctypes.byref(h), None, 0, 0) == mcf.MCF_OK
    assert lib.mcf_plan_update(h, one, 1, None) == mcf.MCF_ERR_SIZE            # created over 0 tensors
    assert lib.mcf_plan_update(h, None, 0, None) == mcf.MCF_OK
    assert lib.mcf_plan_destroy(h) == mcf.MCF_OK
    empty1 = (mcf.Tensor * 1)(mcf.Tensor(None, None, None, None, None, None, 0))
    assert lib.mcf_plan_create(ctypes.byref(h), empty1, 1, 0) == mcf.MCF_OK
    assert lib.mcf_plan_update(h, one, 1, None) == mcf.MCF_ERR_SIZE            # n changed from 0 to 8
    assert lib.mcf_plan_update(h, None, 1, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_plan_update(h, empty1, 1, None) == mcf.MCF_OK
    assert lib.mcf_plan_destroy(h) == mcf.MCF_OK
    empty = (mcf.Tensor * 2)(mcf.Tensor(None, None, None, None, None, None, 0), mcf.Tensor(None, None, None, None, None, None, 0))
    assert lib.mcf_plan_create(ctypes.byref(h), empty, 2, 1) == mcf.MCF_OK
    assert lib.mcf_plan_params(h) == 0
    assert lib.mcf_plan_destroy(h) == mcf.MCF_OK


@pytest.mark.skipif(HAS_GPU, reason="with a device the table allocation succeeds")
def test_plan_create_without_device_reports_hip_error():
    lib = mcf.lib()
    h = ctypes.c_void_p()
    one = (mcf.Tensor * 1)(mcf.Tensor(FAKE, FAKE, FAKE, FAKE, None, FAKE, 8))
    assert lib.mcf_plan_create(ctypes.byref(h), one, 1, 0) == mcf.MCF_ERR_HIP
    assert not h.value


def test_primitive_argument_errors():
    lib = mcf.lib()
    assert lib.mcf_fast2sum(None, FAKE, FAKE, FAKE, 4, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_two_sum(FAKE, FAKE, FAKE, None, 4, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_grow(FAKE, None, FAKE, 4, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_fast2sum(FAKE + 1, FAKE, FAKE, FAKE, 4, None) == mcf.MCF_ERR_ALIGN
    assert lib.mcf_grow(FAKE, FAKE, FAKE, (1 << 35) - 127, None) == mcf.MCF_ERR_SIZE
    assert lib.mcf_fast2sum(None, None, None, None, 0, None) == mcf.MCF_OK
    assert lib.mcf_grow_two_sum(FAKE, FAKE, None, 4, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_two_prod_fma(FAKE, FAKE, FAKE, None, 4, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_scaling(FAKE, FAKE, None, FAKE, FAKE, 4, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_mul(FAKE, FAKE, FAKE, FAKE, FAKE, None, 4, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_mul(FAKE, FAKE, FAKE, FAKE + 1, FAKE, FAKE, 4, None) == mcf.MCF_ERR_ALIGN
    assert lib.mcf_mul(None, None, None, None, None, None, 0, None) == mcf.MCF_OK
    assert lib.mcf_bf16_op(5, FAKE, FAKE, FAKE, 4, None) == mcf.MCF_ERR_VARIANT
    assert lib.mcf_bf16_op(0, FAKE, None, FAKE, 4, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_round_f32(FAKE + 2, FAKE, 4, None) == mcf.MCF_ERR_ALIGN
    assert lib.mcf_round_f32(None, FAKE, 4, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_edq(FAKE, FAKE, None, FAKE, None, 4, FAKE, None, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_edq(FAKE, FAKE, None, FAKE, None, 4, None, None, FAKE) == mcf.MCF_ERR_NULL
    assert lib.mcf_edq(FAKE, FAKE, None, FAKE + 1, None, 4, FAKE, None, FAKE) == mcf.MCF_ERR_ALIGN
    # the component-aware forms: unknown component or code, then the same pointer checks
    assert lib.mcf_primitive(4, 0, FAKE, FAKE, None, None, FAKE, FAKE, 4, None) == mcf.MCF_ERR_VARIANT
    assert lib.mcf_primitive(2, mcf.PRIM_GROW, FAKE, FAKE, None, None, FAKE, FAKE, 4, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_primitive(1, mcf.PRIM_FAST2SUM, FAKE + 1, FAKE, None, None, FAKE, FAKE, 4, None) == mcf.MCF_ERR_ALIGN
    assert lib.mcf_primitive(1, 7, FAKE, FAKE, None, None, FAKE, FAKE, 4, None) == mcf.MCF_ERR_VARIANT
    assert lib.mcf_primitive(1, mcf.PRIM_GROW, FAKE, FAKE, None, None, FAKE, FAKE, 4, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_primitive(1, mcf.PRIM_MUL, FAKE, FAKE, FAKE, FAKE, FAKE, None, 4, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_primitive(1, mcf.PRIM_MUL, FAKE, FAKE, FAKE, FAKE + 1, FAKE, FAKE, 4, None) == mcf.MCF_ERR_ALIGN
    assert lib.mcf_primitive(1, mcf.PRIM_FAST2SUM, None, None, None, None, None, None, 0, None) == mcf.MCF_OK
    assert lib.mcf_component_op(4, 0, FAKE, FAKE, FAKE, 4, None) == mcf.MCF_ERR_VARIANT
    assert lib.mcf_component_op(3, 0, FAKE, None, FAKE, 4, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_component_op(1, 5, FAKE, FAKE, FAKE, 4, None) == mcf.MCF_ERR_VARIANT
    assert lib.mcf_component_op(1, 0, FAKE, None, FAKE, 4, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_round_f32_to(-1, FAKE, FAKE, 4, None) == mcf.MCF_ERR_VARIANT
    assert lib.mcf_round_f32_to(1, FAKE + 2, FAKE, 4, None) == mcf.MCF_ERR_ALIGN
    assert lib.mcf_edq_component(9, FAKE, FAKE, None, FAKE, None, 4, FAKE, None, FAKE) == mcf.MCF_ERR_VARIANT
    assert lib.mcf_edq_component(1, FAKE, FAKE, None, FAKE, None, 4, FAKE, None, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_edq_scratch_bytes(0) >= 16 and lib.mcf_edq_scratch_bytes(1 << 30) > lib.mcf_edq_scratch_bytes(1 << 20)


def test_fp32mw_argument_errors():
    lib = mcf.lib()
    h = ctypes.c_void_p()
    one = (mcf.Fp32Tensor * 1)(mcf.Fp32Tensor(FAKE, FAKE, FAKE, None, FAKE, 8))
    assert lib.mcf_fp32mw_plan_create(ctypes.byref(h), one, 1) == mcf.MCF_ERR_NULL
    bad = (mcf.Fp32Tensor * 1)(mcf.Fp32Tensor(FAKE, FAKE + 2, FAKE, FAKE, FAKE, 8))
    assert lib.mcf_fp32mw_plan_create(ctypes.byref(h), bad, 1) == mcf.MCF_ERR_ALIGN
    assert lib.mcf_fp32mw_plan_create(None, one, 1) == mcf.MCF_ERR_NULL
    hy = _hyper()
    assert lib.mcf_fp32mw_step(None, ctypes.byref(hy), 1, None) == mcf.MCF_ERR_NULL
    assert lib.mcf_fp32mw_plan_create(ctypes.byref(h), None, 0) == mcf.MCF_OK
    assert lib.mcf_fp32mw_step(h, ctypes.byref(hy), 0, None) == mcf.MCF_ERR_STEP
    assert lib.mcf_fp32mw_step(h, ctypes.byref(hy), 3, None) == mcf.MCF_OK
    assert lib.mcf_fp32mw_plan_destroy(h) == mcf.MCF_OK


def test_header_is_plain_c(tmp_path):
    """include/mcf.h must be usable from C (no C++ in the interface)."""
    import shutil
    import subprocess
    if not shutil.which("gcc"):
        pytest.skip("no gcc")
    src = tmp_path / "use_mcf.c"
    src.write_text('#include "mcf.h"\nint main(void) { mcf_hyper h = {1e-3, 0.9, 0.95, 1e-8, 0.1}; (void)h; '
                   'return mcf_status_string(MCF_OK) == 0 || MCF_FMT_FP16 != 0x1000 || MCF_PRIM_MUL != 6; }\n')
    r = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-I", os.path.join(ROOT, "include"), str(src)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_binding_has_every_c_name():
    for n in _declared():
        assert hasattr(mcf, n), n


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_plain_c_consumer_compiles():
    """csrc/abi_demo.c is C99 and needs nothing but the header, the library and the HIP runtime."""
    from paper_2405_03637_amd import build as lib_build
    mcf.lib()                                   # the library it links against is built
    path = lib_build.build_demo()
    assert os.path.exists(path) and os.access(path, os.X_OK)


def test_launch_pacing_and_measurement_aid_argument_errors():
    L = mcf.lib()
    assert L.mcf_set_launch_pacing(129, 0, 0) == mcf.MCF_ERR_SIZE
    assert L.mcf_set_launch_pacing(8, 5000, 0) == mcf.MCF_ERR_SIZE
    assert L.mcf_set_launch_pacing(12, 4, 4) == mcf.MCF_OK
    assert L.mcf_set_launch_pacing(-1, -1, -1) == mcf.MCF_OK          # back to the built-in figures
    vp = ctypes.c_void_p
    one = (vp * 1)(FAKE)
    five = (vp * 5)(*([FAKE] * 5))
    assert L.mcf_stream_mix(one, 1, one, 1, 0, 64, 1, 0, 0, None) == mcf.MCF_OK            # nothing to move
    assert L.mcf_stream_mix(None, 1, one, 1, 64, 64, 1, 0, 0, None) == mcf.MCF_ERR_NULL
    assert L.mcf_stream_mix(one, 1, five, 5, 64, 64, 1, 0, 0, None) == mcf.MCF_ERR_SIZE    # a write needs its read
    assert L.mcf_stream_mix(one, 1, one, 1, 64, 128, 1, 0, 0, None) == mcf.MCF_ERR_VARIANT
    assert L.mcf_stream_mix(one, 1, one, 1, 64, 64, 3, 0, 0, None) == mcf.MCF_ERR_VARIANT
    assert L.mcf_stream_mix(one, 1, one, 1, 24, 64, 1, 0, 0, None) == mcf.MCF_ERR_ALIGN
    assert L.mcf_stream_mix(one, 1, one, 1, 64, 64, 1, 0, 3, None) == mcf.MCF_ERR_VARIANT      # unknown store policy
    odd = (vp * 1)(FAKE + 8)
    assert L.mcf_stream_mix(odd, 1, one, 1, 64, 64, 1, 0, 0, None) == mcf.MCF_ERR_ALIGN
    assert L.mcf_edq_noalloc(0, FAKE, FAKE, None, FAKE, None, (1 << 28) + 1, None, FAKE) == mcf.MCF_ERR_SIZE
    assert L.mcf_edq_noalloc(0, FAKE, FAKE, None, FAKE, None, 16, None, None) == mcf.MCF_ERR_NULL
    assert L.mcf_edq_noalloc(7, FAKE, FAKE, None, FAKE, None, 16, None, FAKE) == mcf.MCF_ERR_VARIANT
