"""Builds libmlfabric_hip.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmlfabric_hip.so")
SOURCES = ["dense.hip", "sparse.hip"]
HEADERS = ["launch.h"]

# -ffp-contract=off: every product and sum is rounded on its own (the results
# are defined bit for bit).  Packed-FP32 instructions are switched off.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fPIC", "-shared", "-Wall", "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build(extra_flags=(), output: str = LIB, verbose: bool = False) -> str:
    """Compile every kernel source into one shared library; returns its path."""
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags,
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", output]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{err}")
    if verbose and err.strip():
        print(err)
    return output


C_CALLER_SRC = os.path.join(ROOT, "tests", "native", "abi_call_cost.c")
C_CALLER = os.path.join(ROOT, "tests", "native", "abi_call_cost")


def build_c_caller() -> str:
    """Compile the plain C program that times the bare C ABI (gcc, linked
    against the built library and the HIP runtime); returns its path."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-O2", "-std=c11", "-D_POSIX_C_SOURCE=199309L", "-Wall",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"), C_CALLER_SRC,
           "-L", HERE, "-lmlfabric_hip", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_1907_00434_amd", "-Wl,-rpath," + os.path.join(rocm, "lib"),
           "-o", C_CALLER]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"gcc failed:\n{res.stderr}")
    return C_CALLER


def is_built() -> bool:
    return os.path.exists(LIB)


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_c_caller())
