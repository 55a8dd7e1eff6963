"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, no GPU code is instrumented):
the library's host precompute as a plain executable, and the oracle's pin tests in a child interpreter that loads a
sanitized build of oracle/s2_oracle.c."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_precompute_under_asan_ubsan(tmp_path):
    if not shutil.which("hipcc"):
        pytest.skip("hipcc not available")
    exe = str(tmp_path / "drv")
    csrc = os.path.join(ROOT, "paper_2505_11157_amd", "csrc")
    cmd = ["hipcc", "-x", "hip", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", csrc,
           os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"), os.path.join(csrc, "s2_grid.cpp"),
           os.path.join(csrc, "s2_trace.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, cwd=str(tmp_path), timeout=600)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:halt_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "sanitize driver ok" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]


def test_oracle_under_asan_ubsan(tmp_path):
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not asan or not os.path.exists(asan):
        pytest.skip("gcc's libasan.so not found")
    lib = str(tmp_path / "liboracle_san.so")
    subprocess.run(["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-fsanitize=address,undefined",
                    "-fno-omit-frame-pointer", "-o", lib, os.path.join(ROOT, "oracle", "s2_oracle.c"), "-lm"], check=True)
    pre = ":".join(x for x in (asan, os.environ.get("LD_PRELOAD", "")) if x)     # the sanitizer runtime goes first
    env = dict(os.environ, LD_PRELOAD=pre, S2_ORACLE_LIB=lib, ASAN_OPTIONS="detect_leaks=0:halt_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1", OMP_NUM_THREADS="4")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_neighbors.py"),
                        os.path.join(ROOT, "tests", "test_oracle_attention.py"), "-k",
                        "not config2_slice"],
                       capture_output=True, text=True, env=env, cwd=ROOT, timeout=1200)
    assert r.returncode == 0 and "passed" in r.stdout, r.stdout[-3000:] + r.stderr[-3000:]
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
