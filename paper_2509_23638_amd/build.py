"""Build the C-ABI library for gfx950 with hipcc (in-tree, no JIT cache)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmoe_hotpath.so")
SOURCES = ["common.hip", "route.hip", "permute.hip", "ffn.hip", "combine.hip", "layer.hip",
           "probe.hip", "stack.hip", "pack.hip", "sched.hip"]
FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
    "-Wall", "-Wno-unused-function",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]
OBJDIR = os.path.join(HERE, "_build")      # object files; not part of the product


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed ({r.returncode}):\n{err}")


def build(verbose: bool = True) -> str:
    """Compile every source (in parallel, one object each: no kernel calls
    device code of another file) and link the shared library."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    # measurement builds only: compile the MOE_TUNE_* kernel-selection overrides in
    flags = FLAGS + (["-DMOE_TUNING"] if os.environ.get("MOE_BUILD_TUNING") == "1" else [])
    os.makedirs(OBJDIR, exist_ok=True)
    objs = [os.path.join(OBJDIR, s.replace(".hip", ".o")) for s in SOURCES]
    jobs = min(len(SOURCES), int(os.environ.get("MAX_JOBS", "8")), os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=max(jobs, 1)) as pool:
        list(pool.map(lambda so: _run([hipcc, *flags, "-c", os.path.join(CSRC, so[0]), "-o", so[1]],
                                      verbose), zip(SOURCES, objs)))
    _run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", *objs, "-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    build()
