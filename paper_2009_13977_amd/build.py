"""Compile the HIP sources into paper_2009_13977_amd/libfasth.so for gfx950.

hipcc cross-compiles without a GPU. The flags disable packed-fp32 instruction
selection (required on the target machines) and build position-independent
device + host code into one shared library with a plain C ABI.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
LIB_PATH = os.path.join(PKG_DIR, "libfasth.so")
SOURCES = [os.path.join(PKG_DIR, "csrc", "fasth.hip")]
HEADERS = [os.path.join(PKG_DIR, "csrc", h) for h in ("fasth_device.h", "fasth_common.h", "fasth_factor.h",
                                                      "fasth_chain.h", "fasth_chain_tile.h", "fasth_chain_pair.h", "fasth_dv.h",
                                                      "fasth_sequential.h", "fasth_peaks.h")]
HEADERS.append(os.path.join(ROOT, "include", "fasth.h"))


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build_library(verbose: bool = True) -> str:
    cmd = [
        hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        # matrix-instruction results stay in the ordinary vector registers: the chain kernel for wide mini-batches
        # uses its accumulators as the next product's operand, and copies between the two register files
        # would cost more than the products' bookkeeping
        "-mllvm", "-amdgpu-mfma-vgpr-form=1",
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG_DIR, "csrc"),
        "-o", LIB_PATH, *SOURCES,
    ]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + "\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB_PATH


def library_is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build_library())
