"""Build libdlm.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libdlm.so")
PEAKS_LIB = os.path.join(HERE, "libdlm_peaks.so")     # achievable-peak micro-benchmarks (bench.py --kernel peaks)
SOURCES = ["core.hip", "commit.hip", "attn.hip", "attn_bwd.hip", "lmhead.hip"]
PEAKS_SOURCES = ["peaks.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + INCLUDE,
         # packed-fp32 code generation off (hipcc-only flag; the host pass warns that it ignores it)
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # "#pragma unroll" must stay a full unroll however long the body gets: the MFMA accumulator arrays
         # are only registers while every index into them is a compile-time constant
         "-mllvm", "-pragma-unroll-threshold=200000",
         "-Wno-unused-command-line-argument"]


def build_lib(verbose: bool = False, save_temps: str | None = None) -> str:
    """Compile every source and link libdlm.so; always recompiles."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "hipcc")
    procs = []
    for src in SOURCES + PEAKS_SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if save_temps:
            cmd.append("-save-temps=obj")
        procs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs, peak_objs = [], []
    for src, obj, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
        (peak_objs if src in PEAKS_SOURCES else objs).append(obj)
    for lib, lib_objs in ((LIB, objs), (PEAKS_LIB, peak_objs)):
        tmp = lib + f".tmp{os.getpid()}"
        subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *lib_objs])
        os.replace(tmp, lib)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True, save_temps="obj" if "--save-temps" in sys.argv else None))
