"""Seeded synthetic parameter sets and gradients, shaped like the paper's models.

This module holds shapes and random-number plumbing only: none of the method's
arithmetic lives here, so both the GPU library's callers and the CPU oracle's
tests may draw their inputs from it.  Values are drawn in fp32 by torch's
seeded generators on the requested device and cast to bf16 by torch
(round-to-nearest-even); a CPU draw and a GPU draw with the same key are
different streams, so a test draws once and copies.

Shapes: GPT and OpenLLaMA layer counts and hidden sizes follow the paper's
model table (App. E, Table 11); hyper-parameters follow Sec. 5 and App. E.2
(beta1 0.9, beta2 0.95 or 0.999, weight decay 0.1).
"""
import torch

# ---- hyper-parameters per workload: (lr, beta1, beta2, eps, weight_decay) ----
HYPER_LIGHT = (3e-4, 0.9, 0.95, 1e-8, 0.1)
HYPER_PLUS_1P3B = (1e-4, 0.9, 0.999, 1e-8, 0.1)
HYPER_STRESS = (2.0 ** -20, 0.9, 0.999, 1e-8, 0.1)

# fp16 components: gradients of size 1e-3 square to 1e-6, below fp16's normal range (2^-14), so the
# synthetic fp16 workloads carry the gradients times a fixed loss scale and epsilon times the same
# factor (Adam's ratio m/sqrt(v) does not depend on the gradient's scale; epsilon does).
FP16_LOSS_SCALE = 1024.0


def fp16_hyper(h):
    lr, b1, b2, eps, wd = h
    return (lr, b1, b2, eps * FP16_LOSS_SCALE, wd)


# FP8 components (3 or 4 significant bits; E4M3 spans 2^-9 .. 448): hyper-parameters that both formats
# hold, or round to something usable -- E4M3 would turn a learning rate of 3e-4 into 0 -- and the same
# loss scale on the gradients.  beta2 = 15/16 is an E4M3 number and, in E5M2, the expansion (1, -1/16).
HYPER_FP8 = (2.0 ** -6, 0.875, 0.9375, 2.0 ** -6, 0.125)


def gpt_shapes(n_layer, d, ffn, vocab, n_pos):
    """GPT-2 style list: embeddings, per-layer {ln1, qkv, proj, ln2, fc, fc2} with biases, final ln."""
    out = [("wte", vocab * d), ("wpe", n_pos * d)]
    for l in range(n_layer):
        p = f"h{l}."
        out += [(p + "ln1.w", d), (p + "ln1.b", d),
                (p + "qkv.w", d * 3 * d), (p + "qkv.b", 3 * d),
                (p + "proj.w", d * d), (p + "proj.b", d),
                (p + "ln2.w", d), (p + "ln2.b", d),
                (p + "fc.w", d * ffn), (p + "fc.b", ffn),
                (p + "fc2.w", ffn * d), (p + "fc2.b", d)]
    out += [("ln_f.w", d), ("ln_f.b", d)]
    return out


def llama_shapes(n_layer, d, ffn, vocab):
    """LLaMA style list: untied embedding and head, RMSNorm vectors, SwiGLU MLP, no biases."""
    out = [("tok_emb", vocab * d)]
    for l in range(n_layer):
        p = f"l{l}."
        out += [(p + "attn_norm", d), (p + "wq", d * d), (p + "wk", d * d), (p + "wv", d * d),
                (p + "wo", d * d), (p + "ffn_norm", d), (p + "w_gate", d * ffn), (p + "w_up", d * ffn),
                (p + "w_down", ffn * d)]
    out += [("final_norm", d), ("lm_head", vocab * d)]
    return out


def _mix(*key):
    """64-bit mix of an integer key tuple (splitmix-style), used only to derive generator seeds."""
    x = 0x9E3779B97F4A7C15
    for k in key:
        x = (x ^ (int(k) & 0xFFFFFFFFFFFFFFFF)) & 0xFFFFFFFFFFFFFFFF
        x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 31
        x = (x * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 29
    return x & 0x7FFFFFFFFFFFFFFF


def _gen(device, *key):
    g = torch.Generator(device=device)
    g.manual_seed(_mix(*key))
    return g


def normal_bf16(n, std, key, device="cpu", mean=0.0, out=None):
    """n draws of N(mean, std^2) in fp32, cast to bf16 (or to out's dtype).  key = tuple of ints."""
    g = _gen(device, *key)
    x = torch.empty(n, dtype=torch.float32, device=device)
    x.normal_(mean=float(mean), std=float(std), generator=g)
    if out is None:
        return x.to(torch.bfloat16)
    out.copy_(x)           # copy_ casts with round-to-nearest-even
    return out


def uniform_f64(n, key):
    """n uniforms in [0,1) on the CPU in fp64 (for per-tensor scales and lengths)."""
    g = _gen("cpu", *key)
    return torch.rand(n, dtype=torch.float64, generator=g)


def stress_shapes(seed=0, total=64 * 1024 * 1024, n_tiny=4096, n_large=64):
    """Precision-stress set: n_tiny tensors of 1..256 elements, interleaved among n_large
    large tensors that share the remainder.  Returns [(name, numel)]."""
    u = uniform_f64(n_tiny, (seed, 5, 1))
    tiny = [1 + int(x * 256) for x in u.tolist()]
    rest = total - sum(tiny)
    base = rest // n_large
    large = [base] * n_large
    large[-1] += rest - base * n_large
    out = []
    per = n_tiny // n_large
    ti = 0
    for k in range(n_large):
        out.append((f"big{k}", large[k]))
        for _ in range(per):
            out.append((f"tiny{ti}", tiny[ti]))
            ti += 1
    while ti < n_tiny:
        out.append((f"tiny{ti}", tiny[ti]))
        ti += 1
    return out


WORKLOADS = {
    # name: (shape list builder, variant, hyper)
    "flat_1m": (lambda: [("flat", 1 << 20)], "light", HYPER_LIGHT),
    "gpt2_125m": (lambda: gpt_shapes(12, 768, 3072, 50257, 1024), "light", HYPER_LIGHT),
    "gpt_1p3b": (lambda: gpt_shapes(24, 2048, 8192, 50304, 2048), "plus", HYPER_PLUS_1P3B),
    "llama_7b": (lambda: llama_shapes(32, 4096, 11008, 32000), "light", HYPER_LIGHT),
    "stress_64m": (lambda: stress_shapes(), "plus", HYPER_STRESS),
}


def shapes(name):
    return WORKLOADS[name][0]()


def total_params(shape_list):
    return sum(n for _, n in shape_list)


def grad_sigmas(name, shape_list, seed=0):
    """Per-tensor gradient standard deviation."""
    if name == "gpt_1p3b":
        u = uniform_f64(len(shape_list), (seed, 3, 2))
        return [10.0 ** (-5.0 + 3.0 * x) for x in u.tolist()]       # log-uniform in [1e-5, 1e-2]
    return [1e-3] * len(shape_list)


def layout(shape_list, misalign_tiny=False, align=8):
    """Element offsets of each tensor inside one flat arena.

    Large tensors start on 16-byte (8-element) boundaries.  With misalign_tiny,
    tensors of at most 256 elements are packed back to back at whatever 2-byte
    offset they land on, which exercises the unaligned head/tail handling;
    align=1 packs every tensor that way."""
    offs = []
    cur = 0
    for _, n in shape_list:
        if not (misalign_tiny and n <= 256):
            cur = (cur + align - 1) // align * align
        offs.append(cur)
        cur += n
    return offs, (cur + 7) // 8 * 8


def init_theta(name, shape_list, offs, arena, seed=0):
    """Fill arena (bf16 or fp16, flat) with the initial parameters of the workload."""
    dev = arena.device
    if name == "stress_64m":
        k = len(shape_list)
        scale = [10.0 ** (-3.0 + 4.0 * x) for x in uniform_f64(k, (seed, 5, 3)).tolist()]
        for i, ((_, n), o) in enumerate(zip(shape_list, offs)):
            g = _gen(dev, seed, 5, 4, i)
            u = torch.rand(n, dtype=torch.float32, device=dev, generator=g)
            sgn = torch.where(torch.rand(n, dtype=torch.float32, device=dev, generator=g) < 0.5, -1.0, 1.0)
            arena[o:o + n].copy_(sgn * scale[i] * (1.0 + 0.5 * u))
        return
    for i, ((_, n), o) in enumerate(zip(shape_list, offs)):
        normal_bf16(n, 0.02, (seed, 0, i), device=dev, out=arena[o:o + n])


def stress_drift(shape_list, offs, arena_len, device, seed=0, sigma=1e-3):
    """Per-element gradient mean of the stress set: sigma/2 with a per-tensor sign (steady drift), fp32."""
    drift = torch.zeros(arena_len, dtype=torch.float32, device=device)
    for i, ((_, n), o) in enumerate(zip(shape_list, offs)):
        drift[o:o + n] = 0.5 * sigma * (1.0 if (_mix(seed, 5, 6, i) & 1) else -1.0)
    return drift


_CHUNK = 1 << 27     # elements drawn per call when filling a whole arena (bounds the fp32 temporary)


def fill_grads(name, shape_list, offs, arena, step, seed=0, sigmas=None, drift=None, grad_scale=1.0):
    """Fill arena (bf16 or fp16, flat) with the gradients of optimizer step `step` (1-based), times grad_scale.

    Sets whose tensors share one sigma are drawn arena-wide (padding between tensors gets values
    too; nobody reads them); the 1.3B set, with a sigma per tensor, is drawn tensor by tensor.
    `drift` (stress set only) is the per-element mean from stress_drift()."""
    dev = arena.device
    if name == "gpt_1p3b":
        if sigmas is None:
            sigmas = grad_sigmas(name, shape_list, seed)
        for i, ((_, n), o) in enumerate(zip(shape_list, offs)):
            normal_bf16(n, sigmas[i] * grad_scale, (seed, 1, step, i), device=dev, out=arena[o:o + n])
        return
    g = _gen(dev, seed, 1, step)
    total = arena.numel()
    for lo in range(0, total, _CHUNK):
        hi = min(total, lo + _CHUNK)
        x = torch.empty(hi - lo, dtype=torch.float32, device=dev)
        x.normal_(mean=0.0, std=1e-3, generator=g)
        if drift is not None:
            x += drift[lo:hi]
        if grad_scale != 1.0:
            x *= grad_scale
        arena[lo:hi].copy_(x)


def expected_totals():
    """Parameter totals the shape lists must reproduce."""
    return {"flat_1m": 1 << 20, "gpt2_125m": 124_439_808, "gpt_1p3b": 1_315_819_520,
            "llama_7b": 6_738_415_616, "stress_64m": 64 * 1024 * 1024}


def bytes_per_param(kind):
    """Algorithmic HBM bytes moved per parameter per step (state read + written, Table 1 turned into traffic)."""
    return {"light": 18, "plus": 22, "kahan": 18, "bf16": 14, "sgd": 14, "fp32mw": 28}[kind]

