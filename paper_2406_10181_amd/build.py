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
           "compress.hip", "api.cpp", "plan.cpp", "reproject.hip", "dense.hip", "fitgrad.hip", "noalloc.hip", "probe.hip"]

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


# Development builds with pieces of the two hot kernels left out (LSP_ABLATE bits, lsp_internal.h): name -> (bits, sources
# to recompile); results of such a library are wrong by design, ablation.py only times it.
ABLATIONS = {
    "a_no_exchange": (0x001, ["compress_gq16_bf16.hip"]), "a_no_staging": (0x002, ["compress_gq16_bf16.hip"]),
    "a_no_batches": (0x004, ["compress_gq16_bf16.hip"]), "a_no_gathers": (0x008, ["compress_gq16_bf16.hip"]),
    "a_no_gathers_no_fmas": (0x018, ["compress_gq16_bf16.hip"]), "a_no_plan_stream": (0x020, ["compress_gq16_bf16.hip"]),
    "a_no_bank_conflicts": (0x040, ["compress_gq16_bf16.hip"]), "a_no_t_store": (0x080, ["compress_gq16_bf16.hip"]),
    "d_no_math": (0x100, ["decompress.hip"]), "d_no_q_loads": (0x200, ["decompress.hip"]), "d_no_u_build": (0x400, ["decompress.hip"]),
    "d_stream_only": (0x700, ["decompress.hip"]), "d_no_bank_conflicts": (0x040, ["decompress.hip"]),
}


def ablation_lib(name: str) -> str:
    return os.path.join(PKG, "ablations", f"liblsp_hip_{name}.so")


def build_ablations(names=None, verbose: bool = False) -> None:
    """Every variant recompiles only the source its switch lives in and links it with the objects of the normal build
    (which must exist: run build() first)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    normal = os.path.join(OBJDIR, "liblsp_hip")
    os.makedirs(os.path.dirname(ablation_lib("x")), exist_ok=True)

    def one(name: str) -> None:
        bits, srcs = ABLATIONS[name]
        objs = []
        for s in SOURCES:
            base = os.path.splitext(s)[0]
            if s in srcs:
                obj = os.path.join(os.path.dirname(ablation_lib(name)), f"{name}_{base}.o")
                cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, f"-DLSP_ABLATE={bits}",
                                               "-x", "hip", "-c", os.path.join(CSRC, s), "-o", obj]
                if verbose:
                    print(" ".join(cmd), flush=True)
                subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
                objs.append(obj)
            else:
                objs.append(os.path.join(normal, base + ".o"))
        subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", ablation_lib(name)])

    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as pool:
        list(pool.map(one, names or list(ABLATIONS)))


PHASE_LIB = os.path.join(PKG, "liblsp_hip_phase.so")   # development build with per-phase cycle counters in kernel A (phase_timing.py)

if __name__ == "__main__":
    if "--ablations" in sys.argv:
        build(incremental=True)
        build_ablations(verbose=True)
    elif "--phase-timing" in sys.argv:
        build(out=PHASE_LIB, defines=("LSP_PHASE_TIMING",), incremental="--incremental" in sys.argv)
    else:
        build(save_temps="--save-temps" in sys.argv, incremental="--incremental" in sys.argv)
