"""Builds the HIP library in-tree with hipcc for gfx950 (cross-compiles without a GPU).

Every source is compiled to an object of its own (in parallel) and the objects are linked into
liblsp_hip.so beside this file."""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "liblsp_hip.so")
OBJDIR = os.path.join(PKG, "_build")
SOURCES = ["compress_gq16_bf16.hip", "compress_gq16_f16.hip", "compress_gq32.hip", "plan_device.hip", "decompress.hip",
           "compress.hip", "api.cpp", "plan.cpp", "reproject.hip", "fitgrad.hip", "noalloc.hip", "probe.hip"]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    "-munsafe-fp-atomics",
    # no packed-fp32 instructions: the compiler would otherwise form them from plain float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build(verbose: bool = True, save_temps: bool = False, out: str = LIB, defines=(), sources=None, jobs: int = 8,
          incremental: bool = False) -> str:
    """incremental: reuse an object that is newer than its source and every header (development only; the default
    compiles everything)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    sources = [s for s in (sources or SOURCES) if os.path.exists(os.path.join(CSRC, s))]
    tag = os.path.splitext(os.path.basename(out))[0]
    objdir = os.path.join(OBJDIR, tag)
    os.makedirs(objdir, exist_ok=True)
    base = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC] + [f"-D{x}" for x in defines]

    def newest_dependency(path: str, seen=None) -> float:
        """Latest modification time of a source and of the project headers it includes, directly or not."""
        seen = set() if seen is None else seen
        if path in seen or not os.path.exists(path):
            return 0.0
        seen.add(path)
        t = os.path.getmtime(path)
        for line in open(path):
            line = line.strip()
            if line.startswith('#include "'):
                name = line.split('"')[1]
                for folder in (CSRC, os.path.join(ROOT, "include")):
                    t = max(t, newest_dependency(os.path.join(folder, name), seen))
        return t

    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > newest_dependency(os.path.join(CSRC, src)):
            return obj
        cmd = base + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if save_temps:
            cmd += ["-save-temps=obj"]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd, cwd=objdir)
        return obj

    with concurrent.futures.ThreadPoolExecutor(max_workers=max(1, min(jobs, len(sources)))) as pool:
        objs = list(pool.map(compile_one, sources))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", out]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.check_call(link, cwd=objdir)
    return out


PHASE_LIB = os.path.join(PKG, "liblsp_hip_phase.so")   # development build with per-phase cycle counters in kernel A (phase_timing.py)

if __name__ == "__main__":
    if "--phase-timing" in sys.argv:
        build(out=PHASE_LIB, defines=("LSP_PHASE_TIMING",), incremental="--incremental" in sys.argv)
    else:
        build(save_temps="--save-temps" in sys.argv, incremental="--incremental" in sys.argv)
