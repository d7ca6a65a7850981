"""Builds libelmo_head.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libelmo_head.so")
SOURCES = [os.path.join(HERE, "csrc", "elmo_head.hip")]
HEADERS = [os.path.join(HERE, "csrc", h) for h in ("numerics.h", "tiles.h", "kernels.h", "topk.h")] + [
    os.path.join(os.path.dirname(HERE), "include", "elmo_head.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed FP32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the update arithmetic rounds after every FP32 operation: no contraction into fused multiply-adds
    "-ffp-contract=off",
    "-Wno-unused-result",
]


def build(verbose: bool = False) -> str:
    """Compile unconditionally; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-o", LIB_PATH, *SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return LIB_PATH


def is_built() -> bool:
    return os.path.exists(LIB_PATH)


if __name__ == "__main__":
    print(build(verbose=True))
