"""The C-ABI's argument-validation layer under AddressSanitizer and UndefinedBehaviorSanitizer
(host only, no GPU): libpkv is built once more with its host code instrumented and a C program
walks every entry point with every class of bad argument.  Validation comes before any launch, so
nothing here needs a device; what the sanitizers watch is the validation code itself (pointer
reads, size products, alignment checks)."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2602_11530_amd", "csrc")


def test_abi_argument_layer_clean_under_sanitizers(tmp_path):
    from paper_2602_11530_amd import build as pkv_build
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    lib = str(tmp_path / "libpkv_san.so")
    flags = [f for f in pkv_build.FLAGS if f != "-O3"] + ["-O1", "-g"]
    subprocess.check_call([pkv_build.HIPCC, *flags, *san, "-o", lib] +
                          [os.path.join(CSRC, s) for s in pkv_build.SOURCES], stderr=subprocess.DEVNULL)
    exe = str(tmp_path / "abi_walk")
    clang = os.path.join(os.path.dirname(os.path.realpath(pkv_build.HIPCC)), "..", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang"
    subprocess.check_call([clang, "-std=c99", "-g", "-O1", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "abi_sanitize_driver.c"), "-o", exe,
                           lib, f"-Wl,-rpath,{tmp_path}", "-Wl,-rpath,/opt/rocm/lib", "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "abi walk: 0 failures" in r.stdout, r.stdout + r.stderr[-3000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
