"""Compile liblsw.so (HIP, gfx950 only) in-tree.  Run as `python -m paper_2405_17741_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "liblsw.so")
SOURCES = [os.path.join(PKG, "csrc", "lsw_api.cpp"), os.path.join(PKG, "csrc", "lsw_kernels.hip")]


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [
        hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU forms
        "-mllvm", "-amdgpu-mfma-vgpr-form",      # matrix-core accumulators in VGPRs: the kernels touch them with VALU ops
        "-Wno-unused-command-line-argument",
        "-Wno-inline-asm",                       # the LDS-DMA helper names M0, a register the compiler reserves, as clobbered
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"),
        "-x", "hip", *SOURCES, "-o", LIB,
    ]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = ("packed-fp32-ops", "warning generated", "warnings generated")
    err = "\n".join(l for l in res.stderr.splitlines() if not any(n in l for n in noise))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
