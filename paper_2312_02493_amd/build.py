"""Builds libartopk.so (gfx950) in-tree with hipcc.  Run as a module or call build()."""

from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libartopk.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # exact IEEE behaviour: no contraction, no fast-math, fp32 denormals kept
    "-ffp-contract=off", "-fno-fast-math", "-fno-gpu-flush-denormals-to-zero",
    # packed fp32 instructions are switched off on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    src = os.path.join(HERE, "csrc", "artopk.hip")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
           src, "-o", LIB_PATH + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        sys.stderr.write(proc.stdout + proc.stderr)
        raise RuntimeError("hipcc failed building libartopk.so")
    if verbose and proc.stderr.strip():
        sys.stderr.write(proc.stderr)
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    build_abi_client(hipcc, verbose)
    return LIB_PATH


ABI_CLIENT_SRC = os.path.join(ROOT, "tests", "abi_client", "abi_client.cpp")
ABI_CLIENT_BIN = os.path.join(ROOT, "tests", "abi_client", "abi_client")


def build_abi_client(hipcc: str, verbose: bool = False) -> str:
    """The plain C++ client of the C ABI that tests/test_gpu_abi_client.py runs (no Python, no PyTorch)."""
    cmd = [hipcc, "-O2", "-std=c++17", "--offload-arch=gfx950", "-I", os.path.join(ROOT, "include"), ABI_CLIENT_SRC,
           "-L", HERE, "-lartopk", "-Wl,-rpath,$ORIGIN/../../paper_2312_02493_amd", "-o", ABI_CLIENT_BIN + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        sys.stderr.write(proc.stdout + proc.stderr)
        raise RuntimeError("hipcc failed building the ABI client")
    os.replace(ABI_CLIENT_BIN + ".tmp", ABI_CLIENT_BIN)
    return ABI_CLIENT_BIN


if __name__ == "__main__":
    print(build(verbose=True))
