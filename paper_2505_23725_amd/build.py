"""Compile the HIP sources in csrc/ into libmuloco.so (gfx950 only), in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libmuloco.so")
MICROBENCH_PATH = os.path.join(HERE, "mlc_microbench")
SOURCES = ["api.hip", "ns_gemm.hip", "ns_chain_small.hip", "inner_elementwise.hip", "outer.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-fno-gpu-rdc", "-ffp-contract=on",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the MuLoCo library needs ROCm to build")
    return exe


def build_library(verbose: bool = True, extra_flags=()) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(HERE, "..", "include"),
           *srcs, "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    build_microbench(verbose)
    return LIB_PATH


def build_microbench(verbose: bool = True) -> str:
    """Achievable-peak microbenchmark (stand-alone executable used by bench.py)."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-Wno-unused-value",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           os.path.join(CSRC, "microbench.hip"), "-o", MICROBENCH_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on microbench.hip:\n" + res.stderr)
    return MICROBENCH_PATH


if __name__ == "__main__":
    print(build_library())
