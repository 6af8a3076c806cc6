"""Builds librpa.so (host C++ + gfx950 HIP kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librpa.so")
LIB_ABLATE = os.path.join(HERE, "librpa_ablate.so")  # measurement build, loaded by ablation.py only
PROBE = os.path.join(HERE, "wide_loop_probe")        # stand-alone measurement program, no part of the library

SOURCES = ["rpa_api.cpp", "rpa_partition.cpp", "rpa_kernels.hip", "rpa_noalloc.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 VALU forms are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA results stay in ordinary VGPRs also in the kernel that needs more than
    # 256 registers (wide, head_dim 256): with the accumulator-register form the
    # compiler copies the whole output accumulator between the two files on every
    # tile.  The other kernels compile identically with and without it.
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    # symbols bind inside the library: the product and the measurement build can
    # be loaded into one process
    "-Wl,-Bsymbolic", "-fvisibility-inlines-hidden",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build_library(verbose: bool = True, extra_flags=(), out: str = LIB) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    cmd = [hipcc(), *FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-x", "hip", *srcs, "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = ("packed-fp32-ops",)
    err = "\n".join(l for l in res.stderr.splitlines() if not any(n in l for n in noise))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + "\n" + res.stderr)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return out


def build_ablation_library(verbose: bool = True) -> str:
    """The same sources with the measurement switches compiled in (rpa_options.ablate)."""
    return build_library(verbose, extra_flags=("-DRPA_ABLATE",), out=LIB_ABLATE)


def build_probe(verbose: bool = True) -> str:
    """The wide kernel's loop without memory traffic as a program of its own
    (csrc/wide_loop_probe.hip): core clocks per tile and sustained clock."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-unused-command-line-argument", os.path.join(CSRC, "wide_loop_probe.hip"), "-o", PROBE]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + "\n" + res.stderr)
    return PROBE


def build_all(verbose: bool = True):
    return [build_library(verbose), build_ablation_library(verbose), build_probe(verbose)]


if __name__ == "__main__":
    print(*build_all(), sep="\n")
