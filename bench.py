#!/usr/bin/env python3
"""Benchmark of the Collage optimizer step on one MI355X.

A step is one pass of the whole path (scalar preparation on the host, then the fused kernel:
moments, bias correction, update, Grow of the parameter expansion) over every parameter of a
LLaMA-7B-shaped set (291 tensors, 6,738,415,616 bf16 parameters), Collage-light, all state
resident in HBM before the timed region.  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama_7b] [--no-extras]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, vendor peak

# HBM traffic per parameter per step as rocprofv3 --pmc measured it (FETCH_SIZE, WRITE_SIZE, each scaled by what the
# same counter reads for a plain copy of known size: FETCH_SIZE x2.0000, WRITE_SIZE x1.0000).  These are NOT measured
# in this run: they are copied from the summaries under profiles/ (the commands are in those files), keyed by the
# full variant name; a variant with no such summary reports null.
PROFILED_TRAFFIC_BYTES_PER_PARAM = {"light": 18.250, "plus": 22.250, "kahan": 18.250, "bf16": 14.250, "sgd": 14.250,
                                    "light+twosum": 18.250, "plus+twosum": 22.250, "light+fp16": 18.250, "plus+fp16": 22.250,
                                    "light+e5m2": 9.125, "light+e4m3": 9.125, "plus+e5m2": 11.125, "fp32mw": 28.250}


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def time_steps(fn, steps, warmup):
    """fn(t) enqueues one step on torch's current stream (the stream the library launches on)."""
    import torch
    for t in range(1, warmup + 1):
        fn(t)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for t in range(warmup + 1, warmup + steps + 1):
        fn(t)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, ev0.elapsed_time(ev1) / 1e3


ROLES = ("theta", "dtheta", "m", "v", "grad", "dv")


def carve(total, count, dev, itemsize=2):
    """One device block holding `count` arenas of `total` 16-bit elements each, back to back at 4 KiB
    multiples.  Every leg of the benchmark steps the same arenas, so the legs differ in the kernel only
    and not in where the allocator happened to put their buffers."""
    import torch
    stride = (total * itemsize + 4095) // 4096 * 4096
    block = torch.zeros(count * stride + 4096, dtype=torch.uint8, device=dev)
    pad = (-block.data_ptr()) % 4096
    return block, [block[pad + i * stride: pad + i * stride + total * itemsize] for i in range(count)]


def build_state(name, variant, arenas):
    """variant: light | plus | bf16 | kahan | sgd, optionally followed by +twosum and/or one of +fp16, +e5m2, +e4m3.
    arenas: six byte arenas from carve(); they are re-initialised (theta drawn, the rest zero) and viewed
    as bf16, fp16 or (their first half) FP8."""
    import torch
    from paper_2405_03637_amd import binding as mcf
    from paper_2405_03637_amd import workloads as W
    shapes = W.shapes(name)
    offs, total = W.layout(shapes, misalign_tiny=(name == "stress_64m"))
    fmt = 1 if "+fp16" in variant else 2 if "+e5m2" in variant else 3 if "+e4m3" in variant else 0
    fp16 = fmt == 1
    base = variant.split("+")[0]
    dtype = (torch.bfloat16, torch.float16, torch.float8_e5m2, torch.float8_e4m3fn)[fmt]
    st = {k: (a if fmt < 2 else a[:total]).view(dtype) for k, a in zip(ROLES, arenas)}
    dev = st["theta"].device
    for k in ROLES:
        st[k].zero_()
    W.init_theta(name, shapes, offs, st["theta"])
    drift = W.stress_drift(shapes, offs, total, dev) if name == "stress_64m" else None
    W.fill_grads(name, shapes, offs, st["grad"], 1, drift=drift, grad_scale=W.FP16_LOSS_SCALE if fmt else 1.0)
    tensors = [(st["theta"][o:o + n], st["dtheta"][o:o + n] if base != "bf16" else None, st["m"][o:o + n],
                st["v"][o:o + n] if base != "sgd" else None,
                st["dv"][o:o + n] if base == "plus" else None, st["grad"][o:o + n]) for (_, n), o in zip(shapes, offs)]
    code = {"light": mcf.LIGHT, "plus": mcf.PLUS, "bf16": mcf.BF16, "kahan": mcf.KAHAN, "sgd": mcf.SGD}[base]
    if "+twosum" in variant:
        code |= mcf.GROW_TWOSUM
    code |= fmt << 12
    plan = mcf.Plan(tensors, code)
    return st, plan, W.total_params(shapes), len(shapes)


def _oracle_rate(name, variant, hyper, n, threads, min_seconds):
    """params/s of the oracle's step over n parameters drawn like the workload's, on `threads` host threads."""
    import numpy as np
    from oracle import oracle as orc
    from paper_2405_03637_amd import workloads as W
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import helpers as H
    theta = H.torch_to_u16(W.normal_bf16(n, 0.02, (0, 0, 0)))
    z = lambda: np.zeros(n, np.uint16)
    dth, m, v, dv = z(), z(), z(), (z() if variant.startswith("plus") else None)
    grads = [H.torch_to_u16(W.normal_bf16(n, 1e-3, (0, 1, t))) for t in (1, 2)]
    code = {"light": orc.LIGHT, "plus": orc.PLUS, "bf16": orc.BF16, "kahan": orc.KAHAN, "sgd": orc.SGD}[variant.split("+")[0]]
    if "+twosum" in variant:
        code |= orc.GROW_TWOSUM
    if "+fp16" in variant:                 # the same bit patterns read as fp16: the oracle's cost does not depend on the values
        code |= orc.STEP_FP16
    if "+e5m2" in variant or "+e4m3" in variant:
        code |= orc.STEP_E5M2 if "+e5m2" in variant else orc.STEP_E4M3
        theta &= 0xFF; grads = [g & 0xFF for g in grads]        # one 8-bit pattern per element
    orc.adamw_step(theta, dth, m, v, dv, grads[0], code, hyper, 1, nthreads=threads)   # warm-up
    steps, t0 = 0, time.perf_counter()
    while steps < 2 or time.perf_counter() - t0 < min_seconds:
        orc.adamw_step(theta, dth, m, v, dv, grads[steps & 1], code, hyper, steps + 2, nthreads=threads)
        steps += 1
    el = time.perf_counter() - t0
    return n * steps / el, steps, el


def cpu_baseline(name, variant, hyper, sample=32 * 1024 * 1024, min_seconds=1.5):
    """The oracle as it stands on the host cores: over the first `sample` parameters of the workload on every
    core the process may use, and on ONE thread over the 2^20-parameter flat tensor of the smallest
    configuration (the per-core figure)."""
    from oracle import oracle as orc
    from paper_2405_03637_amd import workloads as W
    n = min(sample, W.total_params(W.shapes(name)))
    threads = orc.default_threads()
    rate, steps, el = _oracle_rate(name, variant, hyper, n, threads, min_seconds)
    n1 = 1 << 20
    rate1, steps1, el1 = _oracle_rate("flat_1m", variant, hyper, n1, 1, 0.5)
    return {"value": rate, "unit": "params/s", "cores": threads, "kind": "oracle",
            "sample": f"first {n} parameters of {name}, {steps} {variant} steps, {el:.2f} s wall on {threads} threads",
            "per_core": rate / threads,
            "single_thread": {"value": rate1, "unit": "params/s", "cores": 1,
                              "sample": f"flat_1m ({n1} parameters), {steps1} {variant} steps, {el1:.2f} s wall on 1 thread"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama_7b")
    ap.add_argument("--variant", default=None, help="light or plus (default: the workload's own)")
    ap.add_argument("--no-extras", action="store_true", help="skip the plus / fp32-master / copy legs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the step is element-wise and shards with no "
                 "communication); run with --gpus 1")

    import torch
    from paper_2405_03637_amd import binding as mcf
    from paper_2405_03637_amd import workloads as W
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    mcf.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    name = args.workload
    variant = args.variant or W.WORKLOADS[name][1]
    hyper = W.WORKLOADS[name][2]
    if "+fp16" in variant:
        hyper = W.fp16_hyper(hyper)
    if "+e5m2" in variant or "+e4m3" in variant:
        hyper = W.HYPER_FP8

    log(f"bench: building {name} ({variant})")
    _, total = W.layout(W.shapes(name), misalign_tiny=(name == "stress_64m"))
    block, arenas = carve(total, len(ROLES), dev)
    st, plan, n_params, n_tensors = build_state(name, variant, arenas)
    # Bring the device to its steady power/clock state before the W warm-up steps: about a second of
    # plain copies between the two still-zero moment arenas (zeros onto zeros: the optimizer state is
    # untouched).  Without it the first leg measured in a fresh process reads 2-3% slow.
    nb = st["m"].numel() // 8 * 8
    t_end = time.perf_counter() + 1.0
    while time.perf_counter() < t_end:
        for _ in range(8):
            mcf.stream_copy(st["v"][:nb], st["m"][:nb])
        torch.cuda.synchronize()
    wall, gpu_s = time_steps(lambda t: plan.step(hyper, t), args.steps, args.warmup)
    bpp = W.bytes_per_param(variant.split("+")[0]) * (0.5 if ("+e5m2" in variant or "+e4m3" in variant) else 1.0)
    kern_s = gpu_s / args.steps
    achieved = bpp * n_params / kern_s / 1e9
    traffic = PROFILED_TRAFFIC_BYTES_PER_PARAM.get(variant)
    result = {
        "metric": "MCF-AdamW params updated/sec and % of HBM roofline (GB/s) at 7B, 1 GPU",
        "value": n_params * args.steps / wall,
        "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp16" if "+fp16" in variant else "fp8_e5m2" if "+e5m2" in variant else "fp8_e4m3" if "+e4m3" in variant else "bf16",
        "data": "synthetic: theta~N(0,0.02), grad~N(0,1e-3) drawn on the GPU before the timed region; zero-initialised m, v, dtheta",
        "config": {"workload": f"{name} Collage-{variant}: {n_tensors} tensors, {n_params} bf16 params, one launch per step",
                   "params": n_params, "tensors": n_tensors, "variant": variant, "bytes_per_param": bpp},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": (traffic * n_params) if traffic else None,
                     "traffic_source": "rocprofv3 --pmc summaries under profiles/ (not measured in this run)" if traffic else None,
                     "kernel_ms": kern_s * 1e3, "algorithmic_bytes": bpp * n_params},
    }
    extras = {}
    if not args.no_extras:
        try:
            # the same step with the fused EDQ reduction (Def. 3.3) and its two-kernel tail
            edq = torch.zeros(4, dtype=torch.float64, device=dev)
            _, s = time_steps(lambda t: plan.step(hyper, args.warmup + args.steps + t, edq_out=edq), args.steps, 2)
            extras[f"{variant}_with_edq_ms"] = s / args.steps * 1e3
            extras["edq_last"] = edq.cpu().tolist()
        except Exception as e:
            extras["edq_error"] = repr(e)
    plan.destroy()
    if not args.no_extras:
        try:
            # Streaming ceilings measured in this run, on the arenas the step just used.
            # (a) a plain copy of one arena in the step's own launch shape (reads n*2, writes n*2 bytes)
            src, dst = st["theta"], st["dv"]
            nb = src.numel() // 8 * 8
            _, s = time_steps(lambda t: mcf.stream_copy(dst[:nb], src[:nb]), 10, 2)
            extras["copy_GBps"] = 4 * nb * 10 / s / 1e9
            # (b) the same copy in other launch shapes and through the runtime's own device-to-device copy
            shapes_tried = {}
            tag = lambda threads, vec, cap, store: f"{threads}x{vec}" + (f"/cap{cap}" if cap else "") + ("", "/agent", "/agent+nt")[store]
            for threads, vec, cap, store in ((64, 1, 0, 0), (64, 2, 0, 0), (64, 4, 0, 0), (256, 1, 0, 0), (256, 2, 0, 0), (256, 4, 0, 0),
                                             (64, 1, 20, 0), (256, 1, 5, 0), (64, 1, 0, 1), (256, 1, 0, 1), (64, 1, 0, 2), (64, 1, 20, 1)):
                _, s = time_steps(lambda t: mcf.stream_mix([src[:nb]], [dst[:nb]], 2 * nb, threads, vec, cap, store), 6, 2)
                shapes_tried[tag(threads, vec, cap, store)] = round(4 * nb * 6 / s / 1e9, 1)
            extras["copy_shapes_GBps"] = shapes_tried
            extras["copy_best_GBps"] = max(max(shapes_tried.values()), extras["copy_GBps"])
            _, s = time_steps(lambda t: dst[:nb].copy_(src[:nb]), 6, 2)
            extras["hipMemcpyDtoD_GBps"] = 4 * nb * 6 / s / 1e9
            del src, dst
            # (c) the step's own mix of streams with no arithmetic: 5 arenas read, 4 of them written back in place
            rd = [st[k][:nb] for k in ("theta", "dtheta", "m", "v", "grad")]
            mix_tried = {}
            for threads, vec, cap, store in ((64, 1, 6, 0), (64, 1, 10, 0), (64, 1, 0, 0), (256, 2, 0, 0), (64, 1, 8, 1), (64, 1, 10, 1), (64, 1, 11, 1),
                                             (64, 1, 12, 1), (64, 1, 14, 1), (64, 1, 16, 1), (64, 1, 10, 2), (64, 1, 12, 2), (64, 2, 6, 1), (256, 1, 3, 1)):
                _, s = time_steps(lambda t: mcf.stream_mix(rd, rd[:4], 2 * nb, threads, vec, cap, store), 5, 2)
                mix_tried[tag(threads, vec, cap, store)] = round(18 * nb * 5 / s / 1e9, 1)
            extras["stream_5r4w_shapes_GBps"] = mix_tried
            extras["stream_5r4w_GBps"] = max(mix_tried.values())
            # (d) the stand-alone EDQ reduction (Def. 3.3) over whole arenas: five streams read, 24 bytes per 2048 elements written
            scratch = torch.empty(mcf.edq_scratch_bytes(nb) // 8, dtype=torch.float64, device=dev)
            edq4 = torch.zeros(4, dtype=torch.float64, device=dev)
            _, s = time_steps(lambda t: mcf.edq(rd[4], rd[0], rd[1], rd[2], rd[3], scratch, edq4), 5, 2)
            extras["edq_standalone_GBps"] = 10 * nb * 5 / s / 1e9
            extras["edq_standalone_ms"] = s / 5 * 1e3
            del rd, scratch, edq4
            # the other strategies on the same shapes
            for other in ("plus", "light", "kahan", "bf16", "sgd", "light+twosum", "plus+twosum", "light+fp16", "plus+fp16",
                          "light+e5m2", "plus+e5m2", "light+e4m3"):
                if other == variant:
                    continue
                st2, plan2, _, _ = build_state(name, other, arenas)
                h2 = W.HYPER_PLUS_1P3B if other.startswith("plus") else W.HYPER_LIGHT
                if "+fp16" in other:
                    h2 = W.fp16_hyper(h2)
                fp8 = "+e5m2" in other or "+e4m3" in other
                if fp8:
                    h2 = W.HYPER_FP8
                _, s = time_steps(lambda t: plan2.step(h2, t), args.steps, args.warmup)
                extras[f"{other}_GBps"] = W.bytes_per_param(other.split("+")[0]) * (0.5 if fp8 else 1.0) * n_params * args.steps / s / 1e9
                extras[f"{other}_ms"] = s / args.steps * 1e3
                plan2.destroy()
            # option D on the same shapes (separate allocations: measured faster for this mix of 2- and
            # 4-byte streams than one block carved the same way, 29.4-29.6 against 29.8-30.7 ms)
            shapes = W.shapes(name)
            offs, total = W.layout(shapes, misalign_tiny=(name == "stress_64m"))
            st = st2 = arenas = block = None
            torch.cuda.empty_cache()
            th = torch.zeros(total, dtype=torch.bfloat16, device=dev)
            g = torch.zeros_like(th)
            W.init_theta(name, shapes, offs, th)
            W.fill_grads(name, shapes, offs, g, 1)
            master = th.float()
            m32, v32 = torch.zeros_like(master), torch.zeros_like(master)
            plan3 = mcf.Fp32MwPlan([(th[o:o + n], master[o:o + n], m32[o:o + n], v32[o:o + n], g[o:o + n])
                                    for (_, n), o in zip(shapes, offs)])
            _, s = time_steps(lambda t: plan3.step(W.HYPER_LIGHT, t), args.steps, args.warmup)
            extras["fp32mw_GBps"] = W.bytes_per_param("fp32mw") * n_params * args.steps / s / 1e9
            extras["fp32mw_ms"] = s / args.steps * 1e3
            plan3.destroy()
            del master, m32, v32, th, g
        except Exception as e:       # the headline number above stands on its own
            extras["error"] = repr(e)
    st = arenas = block = None
    torch.cuda.empty_cache()
    if extras:
        result["extras"] = extras
        if "copy_best_GBps" in extras:
            result["roofline"]["frac_of_copy"] = achieved / extras["copy_best_GBps"]
        if "stream_5r4w_GBps" in extras and variant.split("+")[0] in ("light", "kahan") and bpp == 18:
            result["roofline"]["frac_of_mix"] = achieved / extras["stream_5r4w_GBps"]

    if not args.no_cpu:
        log("bench: timing the CPU oracle")
        result["cpu_baseline"] = cpu_baseline(name, variant, hyper)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
