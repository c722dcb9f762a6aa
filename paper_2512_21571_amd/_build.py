"""Build the gfx950 shared library in-tree with hipcc (no GPU needed to compile)."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libnnc.so")
SOURCES = ["nnc_kernels.hip", "nnc_decode_mk.hip", "nnc_prefill.hip", "nnc_api.hip", "nnc_plan.cpp"]
HEADERS = [os.path.join(CSRC, "nnc_internal.h"), os.path.join(HERE, "..", "include", "nnc.h")]

OBJ_DIR = os.path.join(HERE, "_build")
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # the compiler may not form packed fp32 instructions on its own
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    # the direct-to-LDS copies set m0 inside inline assembly and list it as clobbered
    "-Wno-inline-asm",
    # k_gemm_prefill_big keeps its accumulators in accumulation registers it names itself in inline
    # assembly: the compiler must never park values of its own there (it would, as a cheaper spill)
    "-mllvm", "-amdgpu-spill-vgpr-to-agpr=0",
]


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def _run(cmd):
    proc = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass reports the packed-fp32 feature as unknown; that is expected
    err = "\n".join(l for l in proc.stderr.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if err.strip():
        print(err)


def build(force: bool = True) -> str:
    """force: compile every source; otherwise only the sources newer than their object file
    (the sources are compiled side by side, one hipcc each, then linked)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    hdr_time = max(os.path.getmtime(h) for h in HEADERS + [os.path.join(CSRC, n) for n in ("nnc_lanes.h", "nnc_half.h", "nnc_plan.h")])
    jobs = []
    for src in SOURCES:
        sp, op = os.path.join(CSRC, src), os.path.join(OBJ_DIR, src + ".o")
        if force or not os.path.exists(op) or os.path.getmtime(op) < max(os.path.getmtime(sp), hdr_time):
            jobs.append(["hipcc", *HIPCC_FLAGS, "-c", "-o", op, sp])
    if jobs or not os.path.exists(LIB_PATH):
        with ThreadPoolExecutor(max_workers=4) as ex:
            list(ex.map(_run, jobs))
        _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] +
             [os.path.join(OBJ_DIR, src + ".o") for src in SOURCES])
    return LIB_PATH


if __name__ == "__main__":
    import sys
    print(build("--stale" not in sys.argv))
