"""Builds libpkv.so (gfx950, hipcc), libpascal_sched.so (host only, g++) and the native
driver program serve_trace in-tree.
``python -m paper_2602_11530_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libpkv.so")
SOURCES = ["pkv_api.hip", "attn_stream.hip", "attn_reduce.hip", "kv_copy.hip", "kv_append.hip",
           "stream_probe.hip"]

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


SCHED_LIB = os.path.join(PKG, "libpascal_sched.so")
SCHED_SOURCES = ["pascal_sched.cpp"]
CXX = os.environ.get("CXX", "g++")
# no fused multiply-add contraction: the QoE measure is compared bit for bit with the checker's
SCHED_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-Wall", "-Wextra"]


def _compile(cmd, out, verbose):
    tmp = out + f".tmp{os.getpid()}"
    cmd = cmd + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, out)
    return out


def build_sched(verbose: bool = True) -> str:
    """The host-side scheduler library: plain C++, no GPU code."""
    return _compile([CXX, *SCHED_FLAGS] + [os.path.join(CSRC, s) for s in SCHED_SOURCES],
                    SCHED_LIB, verbose)


DRIVER = os.path.join(PKG, "serve_trace")


def build_driver(verbose: bool = True) -> str:
    """The native driver program (host code only): links against both libraries."""
    return _compile([HIPCC, "-O2", "-std=c++17", "-Wall", os.path.join(CSRC, "serve_trace.cpp"),
                     "-L", PKG, "-lpkv", "-lpascal_sched", "-Wl,-rpath,$ORIGIN"], DRIVER, verbose)


def build(verbose: bool = True, extra_flags=()) -> str:
    """Compile every source of both libraries and the driver; always recompiles (seconds)."""
    build_sched(verbose)
    lib = _compile([HIPCC, *FLAGS, *extra_flags] + [os.path.join(CSRC, s) for s in SOURCES],
                   LIB, verbose)
    build_driver(verbose)
    return lib


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
