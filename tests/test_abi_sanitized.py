"""The host side of the C ABI (parameter validation, workspace layout, error paths of meda_compress) built with
AddressSanitizer and UndefinedBehaviorSanitizer on the host code and driven by a small native program: 200 000
random parameter sets, valid and invalid, must neither overflow nor read out of bounds.  No GPU is needed: every
call returns before the first kernel launch (the launchers are stubs that abort if reached)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_host_validation_path_under_sanitizers(tmp_path):
    exe = tmp_path / "abi_sanitizer_check"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "native", "abi_sanitizer_check.cpp"),
           os.path.join(ROOT, "paper_2502_17599_amd", "csrc", "meda_api.hip"),
           "-o", str(exe)]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout + run.stderr)[-3000:]
    assert "abi sanitizer check ok" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
