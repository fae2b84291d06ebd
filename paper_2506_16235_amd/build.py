"""Build libnsml.so (HIP kernels for gfx950 + host controller) in-tree with hipcc.

    python -m paper_2506_16235_amd.build

Flags that matter for bit-exact parity with the CPU checker: no fast-math, no fp
contraction (value - code * scale must stay two operations), correctly rounded fp32
divide (hipcc's default), denormals kept (hipcc's default on gfx9).
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(HERE, "libnsml.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off", "-fno-fast-math", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]
# extra hipcc flags for experiments (e.g. "-DNAME"), never needed for a normal build
HIP_FLAGS += os.environ.get("NSML_HIPCC_EXTRA", "").split()
C_FLAGS = ["-O2", "-std=c11", "-fPIC", "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wextra"]


def build(verbose: bool = True) -> str:
    """Compile every source, always (callers decide when a rebuild is needed)."""
    obj_ctl = os.path.join(CSRC, "nsml_ctl.o")
    obj_hip = os.path.join(CSRC, "nsml_kernels.o")
    cmds = [
        ["gcc", *C_FLAGS, "-I", INCLUDE, "-c", os.path.join(CSRC, "nsml_ctl.c"), "-o", obj_ctl],
        [HIPCC, *HIP_FLAGS, "-I", INCLUDE, "-c", os.path.join(CSRC, "nsml_kernels.hip"), "-o", obj_hip],
        [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", obj_ctl, obj_hip, "-o", LIB + ".tmp", "-lm"],
    ]
    for cmd in cmds:
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
    sys.exit(0)
