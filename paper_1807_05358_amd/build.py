"""Builds the HIP library (csrc/ffsim.hip) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "ffsim.hip")
LIB = os.path.join(HERE, "libffsim.so")
DEPS = [SRC] + [os.path.join(HERE, "csrc", h) for h in ("ffsim_kernels.h", "ffsim_chain.h", "ffsim_events.h", "ffsim_strategy.h",
                                                        "ffsim_device.h")] + [
        os.path.join(os.path.dirname(HERE), "include", "ff_sim.h")]

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               # keep the compiler from forming packed-fp32 instructions
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-value"]


def build_library(force: bool = True) -> str:
    """compile libffsim.so; with force=False only if it is missing or older than a source."""
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in DEPS):
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc, *HIPCC_FLAGS, "-o", LIB, SRC])
    return LIB


if __name__ == "__main__":
    print(build_library())
