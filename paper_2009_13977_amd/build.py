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
                                                      "fasth_chain.h", "fasth_chain_tile.h", "fasth_chain_pair.h", "fasth_chain_quad.h", "fasth_chain_team.h", "fasth_chain_teamtile.h", "fasth_dv.h",
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
        # per-kernel register and scratch use, checked below
        "-Rpass-analysis=kernel-resource-usage",
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG_DIR, "csrc"),
        "-o", LIB_PATH, *SOURCES,
    ]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = ("is not a recognized feature for this target", "[-Rpass-analysis=kernel-resource-usage]")
    err = "\n".join(l for l in res.stderr.splitlines() if not any(x in l for x in noise))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + "\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    check_register_use(res.stderr, verbose)
    return LIB_PATH


def check_register_use(remarks: str, verbose: bool = True) -> None:
    """The matrix-core chain kernel is written for results of matrix instructions that stay in the ordinary vector
    registers (`-amdgpu-mfma-vgpr-form=1`, an internal compiler switch): with the switch in effect it uses no
    accumulation registers and no scratch memory. A compiler that accepts the switch but ignores it, or a change
    that pushes the kernel over its register budget, shows here at build time instead of as a slow kernel."""
    import re
    blocks = re.split(r"remark: Function Name: ", remarks)[1:]
    seen = 0
    for b in blocks:
        name = b.split()[0]
        if "chain_tile_kernel" not in name:
            continue
        seen += 1
        agpr = int(re.search(r"AGPRs: (\d+)", b).group(1))
        scratch = int(re.search(r"ScratchSize \[bytes/lane\]: (\d+)", b).group(1))
        if agpr or scratch:
            raise RuntimeError(f"{name}: {agpr} accumulation registers, {scratch} bytes of scratch per lane: "
                               "the matrix-instruction results are not staying in the vector registers")
    if blocks and not seen:
        raise RuntimeError("no chain_tile_kernel in the compiler's resource remarks")
    if verbose and seen:
        print(f"register check: {seen} chain_tile_kernel instantiations, 0 accumulation registers, 0 scratch")


def library_is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build_library())
