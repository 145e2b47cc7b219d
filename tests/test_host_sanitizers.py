"""The host code of libvnm (assignment solver, V/M selection, folding of permutations, size queries,
argument validation) built with AddressSanitizer and UndefinedBehaviorSanitizer and run on the CPU.
Only the host pass of the three sources without device code is compiled, together with
tests/host_sanitize/host_check.cpp, whose stubs stand in for the kernel launchers."""

import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    csrc = os.path.join(ROOT, "paper_2410_16135_amd", "csrc")
    exe = str(tmp_path / "host_check")
    cmd = [hipcc, "--cuda-host-only", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"), "-I", csrc,
           os.path.join(csrc, "vnm_api.hip"), os.path.join(csrc, "vnm_lsa.hip"), os.path.join(csrc, "vnm_select.hip"),
           os.path.join(ROOT, "tests", "host_sanitize", "host_check.cpp"), "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, (run.stdout + run.stderr)[-3000:]
    assert "host_check ok" in run.stdout
    shutil.rmtree(tmp_path, ignore_errors=True)
