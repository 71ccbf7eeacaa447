"""Build librh.so (the HIP library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librh.so")
SOURCES = ["rh_api.hip", "select.hip", "plan.hip", "pack.hip", "unpack.hip", "conv_fp32.hip", "conv_mfma.hip",
           "conv_mfma_duo.hip", "conv_tail.hip", "conv_head.hip", "probe.hip", "temporal.hip"]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-ffp-contract=off",
           "-I" + os.path.join(HERE, "..", "include"), "-I" + CSRC,
           "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed building librh.so")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
