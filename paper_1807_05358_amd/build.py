"""Builds the HIP library for gfx950 with hipcc, in-tree: the host file and the kernel files of
csrc/ are compiled side by side (the kernels are many template instantiations), then linked."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
HOST_UNIT = "ffsim.hip"
KERNEL_UNITS = ["ffsim_k_batch.hip", "ffsim_k_chain.hip", "ffsim_k_try.hip"]   # each compiled per (EXT, GPN)
VARIANTS = [(0, 4), (0, 0), (1, 4), (1, 0), (2, 4), (2, 0)]
UNITS = [HOST_UNIT] + KERNEL_UNITS
HEADERS = ["ffsim_select.h", "ffsim_sweep.h", "ffsim_kernels.h", "ffsim_chain.h", "ffsim_events.h", "ffsim_strategy.h",
           "ffsim_device.h"]
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libffsim.so")
# the same sources with the event loop's section timers compiled in (a diagnostic build: the optional per-candidate
# record then holds clock ticks per section instead of its counters; `bench.py --sections` reads it)
SECTIONS_OBJ_DIR = os.path.join(HERE, "_build_sections")
SECTIONS_LIB = os.path.join(HERE, "libffsim_sections.so")
DEPS = [os.path.join(CSRC, f) for f in UNITS + HEADERS] + [os.path.join(os.path.dirname(HERE), "include", "ff_sim.h")]

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
               # keep the compiler from forming packed-fp32 instructions
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-value"]


def build_library(force: bool = True, sections: bool = False) -> str:
    """compile libffsim.so (sections=True: libffsim_sections.so, the build with section timers);
    with force=False only if it is missing or older than a source."""
    lib_path, obj_dir = (SECTIONS_LIB, SECTIONS_OBJ_DIR) if sections else (LIB, OBJ_DIR)
    extra = ["-DFFSIM_PROFILE"] if sections else []
    if not force and os.path.exists(lib_path) and all(os.path.getmtime(lib_path) >= os.path.getmtime(d) for d in DEPS):
        return lib_path
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(obj_dir, exist_ok=True)
    jobs = [(HOST_UNIT, extra, "ffsim.o")]
    for ext, gpn in VARIANTS:
        for u in KERNEL_UNITS:
            jobs.append((u, [f"-DFFSIM_EXT={ext}", f"-DFFSIM_GPN={gpn}", *extra], f"{os.path.splitext(u)[0]}_e{ext}_g{gpn}.o"))
    objs = [os.path.join(obj_dir, o) for _, _, o in jobs]
    workers = max(1, min(len(jobs), int(os.environ.get("MAX_JOBS", os.cpu_count() or 1))))
    running, failed, todo = [], [], list(zip(jobs, objs))
    while todo or running:
        while todo and len(running) < workers:
            (u, defs, _), obj = todo.pop(0)
            running.append((u + " " + " ".join(defs), subprocess.Popen([hipcc, *HIPCC_FLAGS, *defs, "-c", "-o", obj, os.path.join(CSRC, u)])))
        name, p = running.pop(0)
        if p.wait() != 0:
            failed.append(name)
    if failed:
        raise RuntimeError("hipcc failed on " + ", ".join(failed))
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib_path, *objs])
    return lib_path


if __name__ == "__main__":
    import sys
    print(build_library(sections="--sections" in sys.argv[1:]))
