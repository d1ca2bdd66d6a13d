"""Build the engine's C-ABI library (csrc/*.hip -> csrc/libtent.so) for gfx950 with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(CSRC, "libtent.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # Device code is built without packed-FP32 instruction selection.  The option reaches both passes of
    # hipcc: the gfx950 pass takes it silently, the host (x86) pass does not know the feature and prints
    # "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)" per file, which
    # is harmless.
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB_PATH] + sources()
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
