"""Compile liblsw.so (HIP, gfx950 only) in-tree.  Run as `python -m paper_2405_17741_amd.build`."""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "liblsw.so")
# host code of the C ABI + one translation unit per kernel family
SOURCES = [os.path.join(PKG, "csrc", name) for name in (
    "lsw_api.cpp", "pack_a.hip", "switch_valu.hip", "switch_mfma.hip", "switch_mfma_res.hip", "switch_mfma_bigk.hip",
    "route.hip", "adapter.hip", "probe_inplace.hip", "probe_mfma.hip", "gemv.hip")]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = ("packed-fp32-ops", "warning generated", "warnings generated")
    err = "\n".join(l for l in res.stderr.splitlines() if not any(n in l for n in noise))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build_library(verbose: bool = False) -> str:
    """Every source to an object file (in parallel, under _build/), then one shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [
        "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU forms
        "-mllvm", "-amdgpu-mfma-vgpr-form",      # matrix-core accumulators in VGPRs: the kernels touch them with VALU ops
        "-Wno-unused-command-line-argument",
        "-Wno-inline-asm",                       # the LDS-DMA helper names M0, a register the compiler reserves, as clobbered
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"),
    ]
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = [os.path.join(objdir, os.path.basename(src) + ".o") for src in SOURCES]
    jobs = max(1, min(len(SOURCES), int(os.environ.get("MAX_JOBS", "8"))))
    with concurrent.futures.ThreadPoolExecutor(jobs) as pool:
        list(pool.map(lambda so: _run([hipcc, *flags, "-x", "hip", "-c", so[0], "-o", so[1]], verbose), zip(SOURCES, objs)))
    _run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", *objs, "-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
