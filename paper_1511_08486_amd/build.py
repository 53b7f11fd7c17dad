"""Builds libsfb.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsfb.so")
SOURCES = ["sfb_api.hip", "sfb_forward.hip", "sfb_factor.hip", "sfb_reconstruct.hip", "sfb_sparse.hip", "sfb_bf16.hip",
           "sfb_ssp.hip", "sfb_forward_split.hip", "sfb_reconstruct_split.hip", "sfb_prox.hip", "sfb_reconstruct_small.hip", "sfb_reconstruct_ksplit.hip", "sfb_reconstruct_pair.hip", "sfb_probe.hip", "sfb_fused.hip"]
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-fvisibility=hidden",
    # packed fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def hipcc():
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def build(verbose=False, extra_flags=()):
    """Compile every kernel translation unit and link libsfb.so next to this file."""
    cmd = [hipcc(), *FLAGS, *extra_flags, *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, cwd=CSRC)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
