"""Build step: compile the HIP sources in csrc/ for gfx950 into libsnip_hip.so (in-tree)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libsnip_hip.so")
MICROBENCH = os.path.join(_HERE, "snip_microbench")
SOURCES = ("api.hip", "quant_kernels.hip", "gemm.hip", "gemm_fast.hip", "optim_kernels.hip", "paper_kernels.hip", "gemm_paper.hip")


def build_library(verbose: bool = False) -> str:
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument",
           "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libsnip_hip.so")
    # device microbenchmarks (measured roofline denominators), run by `bench.py --microbench`
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-o", MICROBENCH,
           os.path.join(CSRC, "microbench.hip")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
        raise RuntimeError("hipcc failed building snip_microbench")
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
