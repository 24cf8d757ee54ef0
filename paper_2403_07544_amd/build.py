"""Builds libmammoth_hip.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmammoth_hip.so")
SOURCES = ["runtime.hip", "kernels_pointwise.hip", "kernels_gemm.hip", "kernels_attention.hip",
           "kernels_decode.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-result", "-Wno-unused-value"]


def build(verbose: bool = True, extra_flags=(), out: str = LIB) -> str:
    """extra_flags / out: an experimental build beside the standard one (e.g. a -D switch)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + list(extra_flags) + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    text = "\n".join(l for l in res.stdout.splitlines()
                     if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if verbose and text.strip():
        print(text)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode})\n{res.stdout}")
    return out


if __name__ == "__main__":
    build()
    print("built", LIB)
