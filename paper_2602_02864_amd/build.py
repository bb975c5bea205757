"""Builds libfdc.so (HIP kernels + C ABI) for gfx950 in-tree with hipcc.

    python -m paper_2602_02864_amd.build

hipcc cross-compiles without a GPU.  Packed-FP32 instruction selection is
switched off for all device code.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libfdc.so")
SOURCES = ["fdc_host.cpp", "fdc_api.hip", "gemm_skinny.hip", "gemm_tiled.hip", "rowops.hip", "attention.hip"]

# matrix-instruction accumulators in ordinary VGPRs: the softmax rescales them with
# vector ALU ops, which cannot touch accumulation registers.  The tiled GEMM is the
# opposite case (accumulators only ever feed matrix instructions until the
# epilogue, and there are more of them than VGPRs to spare): it keeps the default.
VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]
NO_VGPR_FORM = {"gemm_tiled.hip"}

HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(" ".join(cmd) + "\n" + r.stdout + r.stderr)
        raise RuntimeError("compilation failed")
    return r


def build(verbose: bool = False, jobs: int = 4) -> str:
    """Compiles every source and links libfdc.so; returns its path."""
    hipcc = _hipcc()
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)

    def one(src):
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc] + HIP_FLAGS + ([] if src in NO_VGPR_FORM else VGPR_FORM) + \
              (["-x", "hip"] if src.endswith(".hip") else []) + \
              ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        _run(cmd)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(one, SOURCES))
    tmp = LIB + ".tmp"
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
