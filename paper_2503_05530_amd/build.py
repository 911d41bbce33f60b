"""Compile the HIP library for gfx950 in-tree: ``python -m paper_2503_05530_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(CSRC, "libproximity.so")

# Keeps the device compiler from forming packed-float32 instructions (v_pk_add/mul/fma_f32) out of ordinary
# float code.  The device pass honours it (tests/test_abi_cpu.py compiles a two-float kernel with and without
# it and looks for those instructions); the host pass of the same command does not know the feature and
# prints "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)", which is harmless
# and left in the build log as it is.
NO_PACKED_FP32 = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
HIPCC_FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-shared", "-fPIC", *NO_PACKED_FP32]


def build_library(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-o", LIB_PATH, os.path.join(CSRC, "proximity.hip")]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    log = proc.stdout
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log)
    return LIB_PATH


if __name__ == "__main__":
    build_library()
    sys.exit(0)
