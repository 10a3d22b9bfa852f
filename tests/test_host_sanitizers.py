"""Host side of libpipeoptim under AddressSanitizer + UndefinedBehaviorSanitizer.

Builds the library's host code with the sanitizers enabled for the host compilation only (the device
code is compiled as usual and never runs here) together with tests/native/host_checks.cpp, and runs the
resulting executable: validation paths, the chunk-table builder and the coefficient derivation must be
free of out-of-bounds accesses, leaks and undefined behaviour.  CPU only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2312_00839_amd", "csrc")


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
def test_host_entry_points_under_asan_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    exe = str(tmp_path / "host_checks")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address,undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(CSRC, "pipeoptim.hip"), os.path.join(CSRC, "step_predict_kernels.hip"),
           os.path.join(CSRC, "near_arena.hip"), os.path.join(CSRC, "static_tables.hip"),
           os.path.join(ROOT, "tests", "native", "host_checks.cpp"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout + run.stderr)[-3000:]
    assert "host checks passed" in run.stdout
