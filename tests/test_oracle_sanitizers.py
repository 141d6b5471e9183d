"""The fp64 checker under AddressSanitizer and UndefinedBehaviorSanitizer (host only).

`oracle/pkv_oracle.c` is compiled once more with `-fsanitize=address,undefined` together with a
small driver that keeps every array in a heap allocation of exactly its size, and run on inputs
made to reach its corners: requests of length 0 and 1, lengths one short of, equal to and one past
a block, unused table entries that point outside the pool, a request whose last block is the last
block of the pool, NaN-poisoned unused slots, empty id lists.  Any access outside an array, any
misaligned or overflowing arithmetic ends the run with a report; the results must equal those of
the ordinary build."""
import os
import struct
import subprocess

import numpy as np
import pytest

import oracle
from paper_2602_11530_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_sanitized")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fno-omit-frame-pointer",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-Wall", "-Wextra", os.path.join(ROOT, "tests", "oracle_sanitize_driver.c"),
                           os.path.join(ROOT, "oracle", "pkv_oracle.c"), "-lm", "-o", exe])
    return exe


def run_case(driver, tmp_path, w, seed, n_ids, n_move):
    rng = np.random.default_rng(seed)
    q, k, v = wl.make_host_tensors(w, poison_unused=True)
    NB, Hkv, B, D = k.shape
    S = w.num_seqs
    ids = rng.permutation(NB)[:n_ids].astype(np.int32)
    ids2 = rng.permutation(NB)[:n_ids].astype(np.int32)
    k_new, v_new = wl.normal_bf16(rng, (S, Hkv, D)), wl.normal_bf16(rng, (S, Hkv, D))
    NB2 = NB + 3
    pool2 = wl.normal_bf16(rng, (NB2, Hkv, B, D))
    msrc = rng.permutation(NB)[:n_move].astype(np.int32)
    mdst = rng.permutation(NB2)[:n_move].astype(np.int32)
    scale_bits = struct.unpack("<I", struct.pack("<f", float(np.float32(w.scale))))[0]
    head = np.array([S, w.num_q_heads, Hkv, D, B, w.max_blocks_per_seq, NB, n_ids, scale_bits,
                     n_move, NB2, 0, 0, 0, 0, 0], dtype=np.int64)
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        for a in (head, q, k, v, w.block_tables, w.context_lens, ids, ids2, k_new, v_new, msrc, mdst, pool2):
            f.write(np.ascontiguousarray(a).tobytes())
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    env.pop("LD_PRELOAD", None)     # the sanitizer runtime must come first in the process
    r = subprocess.run([driver, fin, fout], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0 and "sanitized run ok" in r.stdout, r.stdout + r.stderr
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr
    raw = open(fout, "rb").read()
    off = 0

    def take(dtype, shape):
        nonlocal off
        n = int(np.prod(shape)) * np.dtype(dtype).itemsize
        a = np.frombuffer(raw, dtype=dtype, count=int(np.prod(shape)), offset=off).reshape(shape)
        off += n
        return a

    ref = take(np.float64, (S, w.num_q_heads, D))
    staging = take(np.uint16, (n_ids,) + k.shape[1:])
    scattered = take(np.uint16, k.shape)
    moved = take(np.uint16, pool2.shape)
    k_app, v_app = take(np.uint16, k.shape), take(np.uint16, k.shape)
    assert off == len(raw)
    # the ordinary build on the same inputs
    want = oracle.paged_decode_attn(q, k, v, w.block_tables, w.context_lens, w.scale)
    np.testing.assert_allclose(ref, want, rtol=1e-12, atol=1e-15)
    g = oracle.kv_blocks_gather(k, ids)
    assert np.array_equal(staging, g)
    assert np.array_equal(scattered, oracle.kv_blocks_scatter(g, k, ids2))
    assert np.array_equal(moved, oracle.kv_blocks_move(k, msrc, pool2, mdst))
    ka, va = oracle.kv_append(k_new, v_new, k, v, w.block_tables, w.context_lens)
    assert np.array_equal(k_app, ka) and np.array_equal(v_app, va)


def test_oracle_clean_under_sanitizers_edge_lengths(driver, tmp_path):
    # pool exactly as large as the batch needs: the longest rows end at the pool's last bytes;
    # unused table entries point far outside the pool
    w = wl.custom([0, 1, 15, 16, 17, 31, 32, 33, 255, 256, 257], 8, 2, seed=91, fill=10 ** 6)
    run_case(driver, tmp_path, w, 91, n_ids=7, n_move=5)


def test_oracle_clean_under_sanitizers_tiny_config(driver, tmp_path):
    run_case(driver, tmp_path, wl.cfg1_tiny(), 92, n_ids=0, n_move=0)
    w = wl.custom([600, 1, 48], 12, 3, seed=93, block_size=32, fill=-1)
    run_case(driver, tmp_path, w, 93, n_ids=4, n_move=20)
