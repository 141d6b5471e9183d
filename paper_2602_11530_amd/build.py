"""Builds libpkv.so (gfx950) in-tree with hipcc.  ``python -m paper_2602_11530_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libpkv.so")
SOURCES = ["pkv_api.hip", "attn_stream.hip", "attn_reduce.hip", "kv_copy.hip", "kv_append.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-fno-gpu-rdc",
    # packed fp32 arithmetic is kept off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # keep MFMA accumulators in VGPRs: the softmax rescale touches them with
    # vector ops, and AGPR placement costs a copy each way per block
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def build(verbose: bool = True, extra_flags=()) -> str:
    """Compile every HIP source; always recompiles (seconds)."""
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [HIPCC, *FLAGS, *extra_flags, "-o", tmp] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
