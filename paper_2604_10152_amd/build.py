"""Builds libspecmoe.so (HIP kernels + C ABI) for gfx950, in-tree, with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspecmoe.so")
PEAKS_LIB = os.path.join(HERE, "libspecmoe_peaks.so")     # measurement helpers (bench.py --mode peaks)
PEAKS_SOURCES = ["peaks.hip"]
SOURCES = ["api.hip", "route_topk.hip", "permute.hip", "grouped_swiglu_f32.hip",
           "grouped_swiglu_bf16.hip", "grouped_gemm_bf16_pipe.hip", "grouped_gemm_bf16_pipe16.hip", "combine.hip", "spec_accept.hip", "hot_experts.hip",
           "draft_route.hip", "spec_sample.hip", "pack.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def build(verbose: bool = False) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES + PEAKS_SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        if src in SOURCES:
            objs.append(obj)
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                                            text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        lines = [l for l in out.splitlines() if "not a recognized feature" not in l]
        if p.returncode != 0:
            failed = True
            print(f"[build] {src} FAILED\n" + "\n".join(lines), file=sys.stderr)
        elif verbose and lines:
            print("\n".join(lines))
    if failed:
        raise RuntimeError("hipcc failed")
    tmp = LIB + ".tmp"
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    tmp = PEAKS_LIB + ".tmp"
    pobjs = [os.path.join(objdir, src.replace(".hip", ".o")) for src in PEAKS_SOURCES]
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *pobjs])
    os.replace(tmp, PEAKS_LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
