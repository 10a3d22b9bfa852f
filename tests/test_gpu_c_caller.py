"""The C ABI called from a program that has no Python and no PyTorch in it (tests/native/c_caller.cpp):
plan creation over hipMalloc'ed buffers, the fused call and the prediction-only call on the program's own
stream, every element compared with the CPU oracle linked as a C library; once over hipMalloc'ed buffers, once
over buffers from the library's near-memory arena with the plan localized."""
import os
import subprocess
import sys

import pytest

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "native"))
import build_native  # noqa: E402

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", ["hipMalloc", "arena"])
def test_c_program_calls_the_library_and_matches_the_oracle(oracle, mode):
    exe = build_native.C_CALLER
    if not os.path.exists(exe):                 # run what is built; build only if nothing is
        build_native.build_c_caller()
    print("[gpu-c-caller] running %s (%s)" % (exe, mode), flush=True)
    run = subprocess.run([exe] + (["arena"] if mode == "arena" else []), capture_output=True, text=True, timeout=120)
    print(run.stdout)
    assert run.returncode == 0, (run.stdout + run.stderr)[-3000:]
    assert "c caller ok" in run.stdout
