"""Builds liblagom.so (HIP kernels + host model/search + C ABI) for gfx950, in-tree.

    python -m paper_2602_20656_amd.build

Every translation unit is compiled with floating-point contraction off (the cost model and
the search must round every operation separately to match a plain double-precision
evaluation) and with packed-fp32 instruction selection disabled for device code.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblagom.so")
SOURCES = ["errors.cpp", "cost_model.cpp", "tune.cpp", "model_fill.cpp", "comm_kernel.hip", "gemm.hip", "overlap.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

COMMON = ["-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
          "-Wall", "-Wno-unused-function"]
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = True) -> str:
    objs = []
    build_dir = os.path.join(HERE, "_build")
    os.makedirs(build_dir, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(build_dir, src + ".o")
        cmd = [HIPCC] + COMMON + (DEVICE if src.endswith(".hip") else ["-x", "c++"]) + ["-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"compiling {src} failed:\n{out}")
        if verbose and out.strip():
            print(out)
    link = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    subprocess.check_call(link)
    if verbose:
        print("built", LIB)
    return LIB


def device_assembly(src: str, out_dir: str) -> str:
    """Device-side gfx950 assembly of one kernel source, with the flags of the library build."""
    out = os.path.join(out_dir, os.path.basename(src) + ".gfx950.s")
    cmd = [HIPCC] + COMMON + DEVICE + ["--offload-device-only", "-S", os.path.join(CSRC, src), "-o", out]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return out


if __name__ == "__main__":
    build()
    sys.exit(0)
