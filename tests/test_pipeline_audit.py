"""The LDS hand-over schedules of the two pipelined kernels (tile GEMM: two stages, two stages with early release, one wave per SIMD with the requests between the multiplies, three stages; 256-row attention: K and V
rings) and the tile order, audited on the host: tests/pipeline_audit.cpp instantiates the very templates the kernels
compile (paper_2104_12470_amd/csrc/pipeline.hpp) with a recording executor and checks that no stage is overwritten
while a read of it can be outstanding, that consumed reads see landed tiles, that every K sub-step is multiplied once,
that nothing is in flight at the end, and that planted mistakes are caught."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_lds_handover_schedules_and_tile_order(tmp_path):
    cxx = shutil.which("g++") or shutil.which("c++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = tmp_path / "pipeline_audit"
    subprocess.run([cxx, "-std=c++17", "-O1", "-Wall", "-Wextra", "-Werror", os.path.join(ROOT, "tests", "pipeline_audit.cpp"),
                    "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "all schedules pass" in out.stdout
    assert out.stdout.count("planted mistake caught") == 5
