"""Builds tests/native/c_caller: the C-ABI test program (no Python, no PyTorch in it), linked against the built
libpipeoptim.so and the built oracle library.  hipcc cross-compiles it without a GPU."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
C_CALLER = os.path.join(HERE, "c_caller")


def build_c_caller(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = C_CALLER + ".tmp.%d" % os.getpid()
    cmd = [hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-Wall", "-Wextra",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), C_CALLER + ".cpp", "-o", tmp,
           "-L", os.path.join(ROOT, "paper_2312_00839_amd"), "-lpipeoptim", "-L", os.path.join(ROOT, "oracle"), "-lpo_oracle",
           "-Wl,-rpath,$ORIGIN/../../paper_2312_00839_amd", "-Wl,-rpath,$ORIGIN/../../oracle"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(tmp, C_CALLER)
    return C_CALLER


if __name__ == "__main__":
    print(build_c_caller(verbose=True))
