"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the host code -- CPU only.

Two small drivers under tests/sanitize/ are compiled with -fsanitize=address,undefined and run:
  * the CPU oracle (plain C), every exported routine once on ragged sizes;
  * the library's host side with no GPU present: argument checks, size queries, blob parsing,
    weight re-tiling up to the first device call, and the clean-up after that call fails.  Only
    the host pass of api.hip is instrumented (the device code and the other objects are the
    regular build): that file holds all of the library's host logic.
A sanitizer report or a non-zero status fails the test.  (Device code cannot be run under a
sanitizer here.)
"""
import os
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parents[1]
CLANG = Path("/opt/rocm/lib/llvm/bin/clang++")
HIPCC = Path("/opt/rocm/bin/hipcc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def run_clean(exe):
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300, env=ENV)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out[-3000:]
    assert "Sanitizer" not in out and "runtime error" not in out, out[-3000:]
    return out


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "oracle_driver"
    subprocess.run(["gcc", "-std=gnu99", "-fopenmp", *SAN, "-Wall", "-Wextra",
                    str(ROOT / "tests" / "sanitize" / "oracle_driver.c"), "-o", str(exe), "-lm"], check=True)
    assert "oracle driver ok" in run_clean(exe)


@pytest.mark.skipif(not (CLANG.exists() and HIPCC.exists()), reason="needs the ROCm compilers")
def test_library_host_code_under_asan_and_ubsan(tmp_path):
    from paper_1803_04209_amd import build as hip_build

    objs = [hip_build.BUILD / (Path(s).stem + ".o") for s in hip_build.SOURCES if s != "api.hip"]
    if not all(o.exists() for o in objs):
        hip_build.build_library(verbose=False)
    api_o, drv_o, exe = tmp_path / "api_san.o", tmp_path / "driver.o", tmp_path / "host_api_driver"
    host_san = [f for s in ("-fsanitize=address", "-fsanitize=undefined", "-fno-omit-frame-pointer")
                for f in ("-Xarch_host", s)]
    subprocess.run([str(HIPCC), *[f for f in hip_build.FLAGS if f != "-O3"], "-O1", "-g", *host_san, "-c",
                    str(hip_build.CSRC / "api.hip"), "-o", str(api_o)], check=True, capture_output=True)
    subprocess.run([str(CLANG), "-std=c++17", *SAN, f"-I{hip_build.INCLUDE}", "-c",
                    str(ROOT / "tests" / "sanitize" / "host_api_driver.cpp"), "-o", str(drv_o)], check=True)
    subprocess.run([str(HIPCC), "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                    str(drv_o), str(api_o), *map(str, objs), "-o", str(exe)], check=True, capture_output=True)
    assert "host api driver ok" in run_clean(exe)
