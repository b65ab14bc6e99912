"""The host side of the library under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The library is rebuilt with the sanitizers on its HOST code only (the device code is compiled as usual and never runs
here), a small C++ program (tests/host_sanitize.cpp) drives the buffer manager through thirty thousand requests and
releases and every handle type through creation, every argument check and destruction, and the sanitizers abort on the
first out-of-bounds access, use after free or undefined operation."""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANGXX = "/opt/rocm/llvm/bin/clang++"
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANGXX)), reason="needs the ROCm compilers")
def test_host_code_is_clean_under_asan_and_ubsan():
    out = os.path.join(ROOT, "_build", "sanitize")
    shutil.rmtree(out, ignore_errors=True)
    os.makedirs(out)
    lib = os.path.join(out, "libeet_san.so")
    srcs = sorted(glob.glob(os.path.join(ROOT, "paper_2104_12470_amd", "csrc", "*.hip")))
    host_flags = [f for s in SAN for f in ("-Xarch_host", s)]          # sanitizers on the host pass only
    subprocess.run([HIPCC, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
                    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *host_flags, *srcs, "-o", lib],
                   check=True, capture_output=True)
    exe = os.path.join(out, "host_sanitize")
    subprocess.run([CLANGXX, "-O1", "-g", "-std=c++17", *SAN, os.path.join(ROOT, "tests", "host_sanitize.cpp"),
                    "-L" + out, "-leet_san", "-Wl,-rpath," + out, "-o", exe], check=True, capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and r.stdout.strip() == "ok", (r.returncode, r.stdout[-2000:], r.stderr[-4000:])
