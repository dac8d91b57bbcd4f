"""Builds libmcf_adamw.so (the C-ABI library) in-tree with hipcc for gfx950.

Flags that matter for the arithmetic:
  -ffp-contract=off   no fused multiply-add unless the source writes one (Alg. 6 does)
  -packed-fp32-ops off  keep fp32 arithmetic on the scalar-per-lane VALU instructions
fp32 subnormals are kept (no -fgpu-flush-denormals-to-zero) and '/' and sqrt are the
correctly rounded ones (hipcc's default -fhip-fp32-correctly-rounded-divide-sqrt).
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "mcf_lib.hip")
LIB = os.path.join(HERE, "libmcf_adamw.so")
DEPS = [SRC, os.path.join(HERE, "csrc", "mcf_math.h"), os.path.join(HERE, "csrc", "mcf_host.h"),
        os.path.join(os.path.dirname(HERE), "include", "mcf.h")]


def hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    return "hipcc"


def flags(extra=()):
    return ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wno-unused-command-line-argument", *extra]


def up_to_date():
    return os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(d) for d in DEPS)


def build(force=True, extra=(), out=LIB, verbose=False):
    """Compile the library.  force=False skips the compile when the .so is newer than its sources."""
    if not force and out == LIB and up_to_date():
        return out
    cmd = [hipcc(), *flags(extra), "-o", out, SRC]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.run(cmd, check=True)
    return out


DEMO_SRC = os.path.join(HERE, "csrc", "abi_demo.c")
DEMO = os.path.join(HERE, "mcf_abi_demo")


def build_demo(verbose=False):
    """Compile csrc/abi_demo.c, a plain C99 consumer of the library, with gcc against the HIP runtime."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(rocm, "include"), DEMO_SRC,
           "-L" + HERE, "-lmcf_adamw", "-L" + os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", DEMO]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.run(cmd, check=True)
    return DEMO


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_demo(verbose=True))
