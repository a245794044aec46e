"""The argument-checking layer of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer (host code
only: GPU-side sanitizers are not available). Builds the library once more with the sanitizers on the host
pass, links tests/abi_host_check.cpp against it and runs it; no GPU is needed, every call is refused before
the first GPU call."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
       "-Xarch_host", "-fno-sanitize-recover=undefined"]
COMMON = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", "-mllvm", "-amdgpu-mfma-vgpr-form=1", "-I", os.path.join(ROOT, "include"),
          "-I", os.path.join(ROOT, "paper_2009_13977_amd", "csrc")]


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_argument_checks_under_host_sanitizers(tmp_path):
    lib = tmp_path / "libfasth_san.so"
    exe = tmp_path / "abi_host_check"
    r = subprocess.run(COMMON + SAN + ["-fPIC", "-shared", "-o", str(lib),
                                        os.path.join(ROOT, "paper_2009_13977_amd", "csrc", "fasth.hip")],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    r = subprocess.run(COMMON + SAN + ["-o", str(exe), os.path.join(ROOT, "tests", "abi_host_check.cpp"),
                                        "-L", str(tmp_path), "-lfasth_san", f"-Wl,-rpath,{tmp_path}"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0:protect_shadow_gap=0"  # the HIP runtime reserves address space of its own
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, (r.stdout[-4000:], r.stderr[-4000:])
    assert "abi_host_check: ok" in r.stdout
