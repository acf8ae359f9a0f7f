"""Build the C-ABI library (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdma_hip.so")
PROBE_LIB = os.path.join(HERE, "libdma_probe.so")   # the benchmark's yardsticks: a library of their own
SOURCES = ["api.hip", "mask_gen.hip", "fwd.hip", "bwd.hip", "mask_bwd.hip", "xhead.hip", "decode.hip", "debug_f32.hip"]
PROBE_SOURCES = ["probe.hip"]
# The attention kernels never produce a NaN from finite inputs (inf - inf is avoided explicitly), so
# their max / compare chains may skip NaN canonicalisation; infinities stay honoured (-inf masks).
# With IEEE mode off as well, a maximum is one instruction (no quieting of its inputs first).  The
# device library's helpers are built with the mode on and would not inline into such kernels: these
# two files read launch indices through builtins (wg_id, thread_id) and call no library function.
EXTRA_FLAGS = {"fwd.hip": ["-fno-honor-nans", "-mno-amdgpu-ieee"], "bwd.hip": ["-fno-honor-nans", "-mno-amdgpu-ieee"]}
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-munsafe-fp-atomics", "-Wall", "-Wno-unused-function",
]


def _hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def build_library(verbose=False):
    """Compile every source and link libdma_hip.so (and libdma_probe.so) next to this file.  Always recompiles."""
    hipcc = _hipcc()
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(ln for ln in r.stderr.splitlines() if "packed-fp32-ops" not in ln)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, SOURCES + PROBE_SOURCES))
    for lib, lib_objs in ((LIB, objs[:len(SOURCES)]), (PROBE_LIB, objs[len(SOURCES):])):
        r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *lib_objs, "-o", lib],
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
