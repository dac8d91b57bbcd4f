"""Shared machinery of the GPU parity tests: device arenas for one workload, the plan over them,
seeded sampling of elements, and the oracle run over the sampled elements.

Inputs (initial parameters, per-step gradients) come from paper_2405_03637_amd.workloads drawn on the
GPU by torch; the sampled elements are copied to the host for the oracle.  No oracle input is ever
taken from the library's outputs: the oracle carries its own state for the sampled elements from
step 0 on.  The step is element-wise, so a sampled element's trajectory does not depend on the rest.
"""
import numpy as np
import torch

import helpers as H
from oracle import oracle as orc
from paper_2405_03637_amd import binding as mcf
from paper_2405_03637_amd import workloads as W


def sample_indices(shape_list, offs, full_below=16384, window=2048, n_random=2, seed=0):
    """Arena element indices to check: small tensors entirely; of large ones the first and last
    `window` elements (the unaligned head and the ragged tail) and n_random windows at random,
    deliberately unaligned, offsets."""
    rng = np.random.default_rng(seed)
    parts = []
    for (_, n), o in zip(shape_list, offs):
        if n <= full_below:
            parts.append(np.arange(o, o + n, dtype=np.int64))
            continue
        parts.append(np.arange(o, o + window, dtype=np.int64))
        parts.append(np.arange(o + n - window, o + n, dtype=np.int64))
        for _ in range(n_random):
            s = int(rng.integers(window, n - 2 * window)) | 1
            parts.append(np.arange(o + s, o + s + window, dtype=np.int64))
    return np.unique(np.concatenate(parts))


class Workload:
    """Device state of one named workload and its plan."""

    def __init__(self, name, device="cuda", misalign_tiny=False, seed=0, variant=None, shape_list=None, hyper=None,
                 align=8, fp16=False, fmt=None):
        self.name = name
        self.shapes = shape_list if shape_list is not None else W.shapes(name)
        vname = variant or W.WORKLOADS[name][1]
        self.variant = {"light": mcf.LIGHT, "plus": mcf.PLUS, "bf16": mcf.BF16, "kahan": mcf.KAHAN,
                        "sgd": mcf.SGD, "light+twosum": mcf.LIGHT | mcf.GROW_TWOSUM, "plus+twosum": mcf.PLUS | mcf.GROW_TWOSUM}[vname]
        self.fmt = fmt if fmt is not None else (1 if fp16 else 0)        # component format id, the same in the library and the oracle
        self.fp16 = self.fmt == 1
        self.hyper = hyper or (W.HYPER_FP8 if self.fmt >= 2 else W.fp16_hyper(W.WORKLOADS[name][2]) if self.fp16 else W.WORKLOADS[name][2])
        self.variant |= self.fmt << 12             # the flag bits are the same in the library and the oracle
        self.dtype = (torch.bfloat16, torch.float16, torch.float8_e5m2, torch.float8_e4m3fn)[self.fmt]
        self.offs, self.total = W.layout(self.shapes, misalign_tiny=misalign_tiny, align=align)
        self.seed = seed
        self.device = device
        z = lambda: torch.zeros(self.total, dtype=torch.uint8 if self.fmt >= 2 else self.dtype, device=device).view(self.dtype)
        base = self.variant & 0xFF
        self.theta, self.m = z(), z()
        self.v = z() if base != mcf.SGD else None
        self.dtheta = z() if base != mcf.BF16 else None
        self.dv = z() if base == mcf.PLUS else None
        self.grad = z()
        W.init_theta(name, self.shapes, self.offs, self.theta, seed=seed)
        self.drift = W.stress_drift(self.shapes, self.offs, self.total, device, seed) if name == "stress_64m" else None
        self.sigmas = W.grad_sigmas(name, self.shapes, seed)
        tensors = []
        for (_, n), o in zip(self.shapes, self.offs):
            sl = slice(o, o + n)
            tensors.append((self.theta[sl], self.dtheta[sl] if self.dtheta is not None else None, self.m[sl],
                            self.v[sl] if self.v is not None else None,
                            self.dv[sl] if self.dv is not None else None, self.grad[sl]))
        self.plan = mcf.Plan(tensors, self.variant)
        self.n_params = W.total_params(self.shapes)
        assert self.plan.params == self.n_params

    def state_names(self):
        return ["theta"] + (["dtheta"] if self.dtheta is not None else []) + ["m"] + (["v"] if self.v is not None else []) + \
            (["dv"] if self.dv is not None else [])

    def new_grads(self, step):
        W.fill_grads(self.name, self.shapes, self.offs, self.grad, step, seed=self.seed, sigmas=self.sigmas,
                     drift=self.drift, grad_scale=W.FP16_LOSS_SCALE if self.fmt else 1.0)

    def gather(self, tensor, idx_dev):
        if tensor.element_size() == 1:
            tensor = tensor.view(torch.uint8)           # index the patterns, not a float8 tensor
        return H.torch_to_u16(tensor[idx_dev])

    def close(self):
        self.plan.destroy()


class SampledOracle:
    """Oracle state for the sampled elements of a Workload, advanced in lock-step."""

    def __init__(self, wl, idx):
        self.wl = wl
        self.idx = idx
        self.idx_dev = torch.from_numpy(idx).to(wl.device)
        self.state = {k: wl.gather(getattr(wl, k), self.idx_dev) for k in wl.state_names()}
        # dtheta, m, v, dv start at zero by construction; theta is the generator's draw
        for k in wl.state_names():
            if k != "theta":
                assert not self.state[k].any()

    def step(self, t, want_delta=False):
        g = self.wl.gather(self.wl.grad, self.idx_dev)
        s = self.state
        delta = np.empty(g.size, np.uint16) if want_delta else None
        orc.adamw_step(s["theta"], s.get("dtheta"), s["m"], s.get("v"), s.get("dv"), g, self.wl.variant, self.wl.hyper, t,
                       delta_out=delta)
        return delta

    def mismatches(self):
        """{state name: number of sampled elements whose bits differ from the device}."""
        out = {}
        for k in self.wl.state_names():
            dev = self.wl.gather(getattr(self.wl, k), self.idx_dev)
            out[k] = int(np.count_nonzero(dev != self.state[k]))
        return out


def assert_bitwise(mism, where):
    assert all(v == 0 for v in mism.values()), f"{where}: mismatching elements {mism}"


def full_oracle_run(wl, steps, edq=False, check_each=True):
    """Whole-state comparison after every step, oracle over every element."""
    names = wl.state_names()
    host = {k: H.torch_to_u16(getattr(wl, k)) for k in names}
    edq_dev = torch.zeros(4, dtype=torch.float64, device=wl.device) if edq else None
    live = np.zeros(wl.total, bool)
    for (_, n), o in zip(wl.shapes, wl.offs):
        live[o:o + n] = True
    for t in range(1, steps + 1):
        wl.new_grads(t)
        g = H.torch_to_u16(wl.grad)
        before = {k: host[k].copy() for k in ("theta", "dtheta") if k in host} if edq else None
        delta = np.zeros(wl.total, np.uint16) if edq else None
        # the oracle steps the whole arena; padding between tensors is stepped too and then ignored
        orc.adamw_step(host["theta"], host.get("dtheta"), host["m"], host.get("v"), host.get("dv"), g, wl.variant, wl.hyper, t,
                       delta_out=delta)
        wl.plan.step(wl.hyper, t, edq_out=edq_dev)
        torch.cuda.synchronize()
        if check_each or t == steps:
            for k in names:
                dev = H.torch_to_u16(getattr(wl, k))
                bad = np.flatnonzero((dev != host[k]) & live)
                assert bad.size == 0, f"{wl.name} step {t} {k}: {bad.size} mismatches, first at {int(bad[0])}: " \
                                      f"got {dev[bad[0]]:#06x} want {host[k][bad[0]]:#06x}"
                # padding is never written by the library
                assert not dev[~live].any()
                host[k][~live] = 0
        if edq:
            acc = orc.EdqAccumulator(fmt=wl.fmt)
            for (_, n), o in zip(wl.shapes, wl.offs):
                sl = slice(o, o + n)
                d0 = before["dtheta"][sl].copy() if "dtheta" in host else None
                d1 = host["dtheta"][sl].copy() if "dtheta" in host else None
                acc.add(delta[sl].copy(), before["theta"][sl].copy(), d0, host["theta"][sl].copy(), d1)
            want = acc.value()
            got = edq_dev.cpu().numpy()
            assert abs(got[0] - want) <= 1e-5 * abs(want), (t, got, want)
            assert int(got[3]) == acc.lost.value, (t, got[3], acc.lost.value)          # exact integer
            assert abs(got[1] - acc.s1.value) <= 1e-5 * abs(acc.s1.value) and abs(got[2] - acc.s2.value) <= 1e-5 * acc.s2.value
            assert want > 0


# ------------------------------------------------------------------ whole-state comparisons at the large sets
class HostMirror:
    """A pinned host buffer that device arenas of 16-bit patterns are fetched into (reused call after call)."""

    def __init__(self, n):
        self.buf = torch.empty(n, dtype=torch.int16, pin_memory=True)
        self.np = self.buf.numpy().view(np.uint16)

    def fetch(self, t):
        """Bit patterns of the 16-bit device tensor t; the returned array is a view that the next fetch overwrites."""
        n = t.numel()
        self.buf[:n].copy_(t.view(torch.int16))
        return self.np[:n]


def same_bits(a, b):
    """Whether two uint16 arrays hold the same patterns (compared eight bytes at a time where they can be)."""
    assert a.shape == b.shape and a.dtype == np.uint16 and b.dtype == np.uint16
    n4 = a.size // 4 * 4
    if a.ctypes.data % 8 == 0 and b.ctypes.data % 8 == 0 and a.flags["C_CONTIGUOUS"] and b.flags["C_CONTIGUOUS"]:
        if not np.array_equal(a[:n4].view(np.uint64), b[:n4].view(np.uint64)):
            return False
        return np.array_equal(a[n4:], b[n4:])
    return np.array_equal(a, b)


def describe_mismatch(got, want, shapes, offs):
    """Where two arenas differ: tensor, element, patterns (called only after same_bits said no)."""
    for (name, n), o in zip(shapes, offs):
        bad = np.flatnonzero(got[o:o + n] != want[o:o + n])
        if bad.size:
            i = int(bad[0])
            return f"tensor {name} (n={n}): {bad.size} elements differ, first at {i}: got {got[o + i]:#06x} want {want[o + i]:#06x}"
    return "the padding between tensors differs (the library must not write there)"


def zero_gaps(arr, shapes, offs):
    """The oracle steps a whole arena, padding between tensors included; the library never touches padding."""
    cur = 0
    for (_, n), o in zip(shapes, offs):
        if o > cur:
            arr[cur:o] = 0
        cur = o + n
    if cur < arr.size:
        arr[cur:] = 0


def edq_over_tensors(delta, th0, dth0, th1, dth1, shapes, offs, fmt, pool, piece=1 << 23):
    """The oracle's EDQ totals over every tensor of an arena: the oracle's own accumulation on pieces of
    at most `piece` elements, run side by side on the host cores, and the partial totals added in fp64."""
    jobs = []
    for (_, n), o in zip(shapes, offs):
        for lo in range(o, o + n, piece):
            jobs.append((lo, min(o + n, lo + piece)))

    def one(job):
        lo, hi = job
        acc = orc.EdqAccumulator(fmt=fmt)
        acc.add(delta[lo:hi], th0[lo:hi], None if dth0 is None else dth0[lo:hi], th1[lo:hi], None if dth1 is None else dth1[lo:hi])
        return acc.s1.value, acc.s2.value, acc.lost.value

    parts = list(pool.map(one, jobs))
    total = orc.EdqAccumulator(fmt=fmt)
    total.s1.value = float(np.sum(np.array([p[0] for p in parts], np.float64)))
    total.s2.value = float(np.sum(np.array([p[1] for p in parts], np.float64)))
    total.lost.value = int(sum(p[2] for p in parts))
    return total


def whole_state_run(wl, steps, check_at, say, edq_every_step=False, on_grads=None):
    """The oracle over EVERY element of the workload for `steps` steps, beside the library: all state
    tensors compared bit for bit at the steps in check_at, and (edq_every_step) the fused EDQ outputs
    compared with the oracle's at every step.  Gradients are drawn on the device and fetched; no oracle
    input comes from the library's results.  on_grads(t) is called once step t's gradients are on the device and
    before the library steps (for a caller that follows sampled elements of its own in lock-step)."""
    from concurrent.futures import ThreadPoolExecutor
    names = wl.state_names()
    mirror = HostMirror(wl.total)
    host = {k: mirror.fetch(getattr(wl, k)).copy() for k in names}
    has_dth = "dtheta" in host
    before = {k: np.empty_like(host[k]) for k in ("theta", "dtheta") if k in host} if edq_every_step else None
    delta = np.zeros(wl.total, np.uint16) if edq_every_step else None
    edq_dev = torch.zeros(4, dtype=torch.float64, device=wl.device) if edq_every_step else None
    pool = ThreadPoolExecutor(max_workers=orc.default_threads()) if edq_every_step else None
    for t in range(1, steps + 1):
        wl.new_grads(t)
        if on_grads is not None:
            on_grads(t)
        g = mirror.fetch(wl.grad)
        if edq_every_step:
            for k in before:
                np.copyto(before[k], host[k])
        wl.plan.step(wl.hyper, t, edq_out=edq_dev)                 # the device works while the oracle does
        orc.adamw_step(host["theta"], host.get("dtheta"), host["m"], host.get("v"), host.get("dv"), g, wl.variant, wl.hyper, t,
                       delta_out=delta)
        if edq_every_step:
            acc = edq_over_tensors(delta, before["theta"], before.get("dtheta"), host["theta"], host.get("dtheta"),
                                   wl.shapes, wl.offs, wl.fmt, pool)
            want = acc.value()
            got = edq_dev.cpu().numpy()
            assert abs(got[0] - want) <= 1e-5 * abs(want), (t, got, want)
            assert int(got[3]) == acc.lost.value, (t, got[3], acc.lost.value)            # an exact integer
            assert abs(got[1] - acc.s1.value) <= 1e-5 * abs(acc.s1.value) and abs(got[2] - acc.s2.value) <= 1e-5 * acc.s2.value
            assert want > 0
        if t in check_at:
            torch.cuda.synchronize()
            for k in names:
                zero_gaps(host[k], wl.shapes, wl.offs)
                dev = mirror.fetch(getattr(wl, k))
                assert same_bits(dev, host[k]), f"{wl.name} step {t} {k}: " + describe_mismatch(dev, host[k], wl.shapes, wl.offs)
            # the step ran everywhere (the comparison above says so element by element; this is the cheap cross-check
            # the sampled runs rely on): m is non-zero except where a gradient was drawn as exactly zero or, later,
            # where a moment cancelled exactly -- about one element in a thousand with 8-bit significands
            moved = int(torch.count_nonzero(wl.m).item())
            assert 0.99 * wl.n_params <= moved <= wl.n_params, f"{wl.name} step {t}: m is non-zero at {moved} of {wl.n_params} elements"
            say(f"{wl.name}: step {t}: every element of {', '.join(names)} identical ({wl.n_params} parameters)"
                + (f", EDQ {got[0]:.9e} (oracle {want:.9e}), lost {int(got[3])}" if edq_every_step else ""))
        elif edq_every_step:
            say(f"{wl.name}: step {t}: EDQ {got[0]:.9e} (oracle {want:.9e}), lost {int(got[3])}")
    if pool is not None:
        pool.shutdown()
    return host


def streamed_whole_state_check(wl, theta0, grads, snapshots, say, piece=1 << 25):
    """Every element of a set too large to mirror on the host, piece by piece.  theta0: the initial parameters
    (device copy taken before the first step); grads[t-1]: the gradient arena of step t, kept on the device;
    snapshots[t-1]: {name: device arena} of the library's state after step t.  The oracle starts every piece from
    (theta0, zeros) and runs the len(grads) steps, comparing all state tensors after each.  Returns the number
    of elements compared."""
    names = wl.state_names()
    mirrors = {k: HostMirror(piece) for k in ["theta0"] + [f"g{t}" for t in range(len(grads))] + names}
    work = {k: np.zeros(piece, np.uint16) for k in names}
    done = 0
    for ti, ((name, n), o) in enumerate(zip(wl.shapes, wl.offs)):
        for lo in range(o, o + n, piece):
            hi = min(o + n, lo + piece)
            k = hi - lo
            st = {}
            for s in names:
                st[s] = work[s][:k]
                st[s][:] = 0
            np.copyto(st["theta"], mirrors["theta0"].fetch(theta0[lo:hi]))
            for t, (g_dev, snap) in enumerate(zip(grads, snapshots), start=1):
                g = mirrors[f"g{t - 1}"].fetch(g_dev[lo:hi])
                orc.adamw_step(st["theta"], st.get("dtheta"), st["m"], st.get("v"), st.get("dv"), g, wl.variant, wl.hyper, t)
                for s in names:
                    dev = mirrors[s].fetch(snap[s][lo:hi])
                    if not same_bits(dev, st[s]):
                        bad = np.flatnonzero(dev != st[s])
                        raise AssertionError(f"{wl.name} step {t} {s}, tensor {name}: {bad.size} elements differ in [{lo - o}, {hi - o}), "
                                             f"first at {lo - o + int(bad[0])}: got {dev[bad[0]]:#06x} want {st[s][bad[0]]:#06x}")
            done += k
        if ti % 32 == 31 or ti == len(wl.shapes) - 1:
            say(f"{wl.name}: {ti + 1} of {len(wl.shapes)} tensors, {done} elements, identical after each of {len(grads)} steps")
    return done
