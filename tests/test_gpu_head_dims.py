"""Head dimensions 64 and 256 (128 is what every other test uses): same parity bar, same edge
cases.  The operand layouts of the stream kernel differ per head dimension (V loads of 8 bytes
and four output tiles at 64; two 128-dim halves, sixteen tiles and one wavefront per SIMD at
256), so the sweep of lengths, group sizes and partitions is repeated for each."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_11530_amd import binding as pkv
from paper_2602_11530_amd import workloads as wl

from gpu_util import (MAX_ABS, REL_L2, abs_error_within_bar, assert_launchable, run_attn, run_attn_dev,
                      shape_of, to_bits, to_dev)

pytestmark = pytest.mark.gpu

EDGE = [1, 15, 16, 17, 31, 32, 33, 0, 2, 255, 256, 257, 511, 512, 513, 1000, 3, 4999, 5001]
SHAPES = {64: [(40, 8), (8, 2), (16, 1), (7, 7), (12, 4)],
          256: [(40, 8), (8, 2), (8, 1), (7, 7), (12, 4)]}     # G <= 8 at D = 256


def check(w, q, k, v, got, what):
    ref = oracle.paged_decode_attn(q, k, v, w.block_tables, w.context_lens, w.scale)
    c = oracle.compare(got, ref)
    print(f"{what}: {c}", flush=True)
    assert np.isfinite(wl.bf16_bits_to_f64(got)).all()
    assert c["rel_l2"] <= REL_L2 and c["worst_seq_rel_l2"] <= 2 * REL_L2, c
    assert abs_error_within_bar(got, ref), c       # one- to three-token requests are in the batch


@pytest.mark.parametrize("D", [64, 256])
@pytest.mark.parametrize("P", [0, 64, 512])
def test_edge_lengths(device, D, P):
    for hq, hkv in SHAPES[D]:
        w = wl.custom(EDGE, hq, hkv, seed=800 + D + hq, num_pool_blocks=900, partition_size=P,
                      head_dim=D)
        assert w.q_shape()[2] == D and w.pool_shape()[3] == D and w.scale == np.float32(D ** -0.5)
        q, k, v = wl.make_host_tensors(w, poison_unused=True)
        print(f"D={D} P={P} hq={hq} hkv={hkv}", flush=True)
        got = run_attn(w, q, k, v)
        check(w, q, k, v, got, f"D={D} hq={hq} hkv={hkv} P={P}")
        assert not got.reshape(w.q_shape())[EDGE.index(0)].any()


@pytest.mark.parametrize("D", [64, 256])
def test_closed_forms(device, D):
    """A one-token context returns its V row bit for bit; V = 1 returns exactly 1; a zero scale
    returns the mean of the valid V rows, unmoved by the poison in the unused slots."""
    lens = [1, 1, 300, 77, 16, 1]
    w = wl.custom(lens, 16, 4, seed=31 + D, num_pool_blocks=64, head_dim=D)
    q, k, v = wl.make_host_tensors(w, poison_unused=True)
    got = run_attn(w, q, k, v).reshape(w.q_shape())
    for s, L in enumerate(lens):
        if L == 1:
            for h in range(16):
                assert np.array_equal(got[s, h], v[w.block_tables[s, 0], h // 4, 0])
    ones = np.where(v == wl.BF16_INF, v, np.uint16(0x3F80))
    got = run_attn(w, q, k, ones)
    assert (got == 0x3F80).all()
    got = run_attn(w, q, k, v, scale=0.0)
    ref = oracle.paged_decode_attn(q, k, v, w.block_tables, w.context_lens, 0.0)
    c = oracle.compare(got, ref)
    assert c["max_abs"] <= MAX_ABS and c["rel_l2"] <= REL_L2, c


@pytest.mark.parametrize("D", [64, 256])
def test_paging_and_partition_invariance(device, D):
    """Permuting the physical blocks (tables rewritten) leaves every bit unchanged; the partition
    size moves the result only within the tolerance."""
    lens = [1300, 77, 2048, 640, 33, 4100]
    w = wl.custom(lens, 40, 8, seed=5, head_dim=D)
    q, k, v = wl.make_host_tensors(w)
    base = run_attn(w, q, k, v)
    rng = np.random.default_rng(9)
    perm = rng.permutation(w.num_pool_blocks).astype(np.int32)     # old id -> new id
    k2, v2 = np.empty_like(k), np.empty_like(v)
    k2[perm], v2[perm] = k, v
    w2 = wl.custom(lens, 40, 8, seed=5, head_dim=D)
    w2.block_tables = np.where(w.block_tables >= 0, perm[np.maximum(w.block_tables, 0)], -1).astype(np.int32)
    assert np.array_equal(run_attn(w2, q, k2, v2), base)
    ref = oracle.paged_decode_attn(q, k, v, w.block_tables, w.context_lens, w.scale)
    for P in (16, 128, 512, 4096):
        c = oracle.compare(run_attn(w, q, k, v, partition_size=P), ref)
        assert c["max_abs"] <= MAX_ABS and c["rel_l2"] <= REL_L2, (P, c)


@pytest.mark.parametrize("D", [64, 256])
def test_append_then_attend(device, D):
    final = np.array([20, 32, 33, 515, 1300, 3], np.int32)
    w = wl.custom(final, 40, 8, seed=90 + D, num_pool_blocks=160, head_dim=D)
    rng = np.random.default_rng(D)
    q, k, v = wl.make_host_tensors(w)
    k_d, v_d, t_d = to_dev(k), to_dev(v), to_dev(w.block_tables)
    k_h, v_h = k.copy(), v.copy()
    for back in (2, 1, 0):
        w.context_lens = final - back
        assert_launchable(w)
        k_new = wl.normal_bf16(rng, (w.num_seqs, 8, D))
        v_new = wl.normal_bf16(rng, (w.num_seqs, 8, D))
        q = wl.normal_bf16(rng, w.q_shape())
        lens_d = to_dev(w.context_lens)
        pkv.kv_append(to_dev(k_new), to_dev(v_new), k_d, v_d, t_d, lens_d, shape_of(w))
        out = run_attn_dev(w, to_dev(q), k_d, v_d, t_d, lens_d)
        torch.cuda.synchronize()
        k_h, v_h = oracle.kv_append(k_new, v_new, k_h, v_h, w.block_tables, w.context_lens)
        assert np.array_equal(to_bits(k_d), k_h) and np.array_equal(to_bits(v_d), v_h)
        check(w, q, k_h, v_h, to_bits(out), f"D={D} append step -{back}")


@pytest.mark.parametrize("D", [64, 256])
def test_config2_lengths_at_this_head_dim(device, D):
    """The Qwen-32B-shaped batch (64 requests, U{1024..8192}, 40 query / 8 KV heads) with this head
    dimension: full oracle parity, and the bandwidth it streams at."""
    w = wl.cfg2_qwen32b(head_dim=D)
    assert_launchable(w)
    g = torch.Generator(device=device)
    g.manual_seed(w.seed + 17)
    q = torch.randn(w.q_shape(), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    k = torch.randn(w.pool_shape(), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn(w.pool_shape(), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    t_d, l_d = to_dev(w.block_tables), to_dev(w.context_lens)
    mc = int(w.context_lens.max())
    out = run_attn_dev(w, q, k, v, t_d, l_d, max_context_len=mc)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    shape = shape_of(w, None, mc)
    ws = torch.empty(pkv.pkv_attn_workspace_bytes(shape), dtype=torch.uint8, device=device)
    reps = 20
    a.record()
    for _ in range(reps):
        pkv.paged_decode_attn(q, k, v, t_d, l_d, float(w.scale), out, shape, ws)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / reps
    print(f"D={D}: {w.attn_algorithmic_bytes() / 1e9:.3f} GB in {ms:.4f} ms = "
          f"{w.attn_algorithmic_bytes() / ms / 1e6:.0f} GB/s", flush=True)
    check(w, to_bits(q), to_bits(k), to_bits(v), to_bits(out), f"cfg2 lengths at D={D}")


@pytest.mark.parametrize("case", range(36))
def test_random_shapes_all_variants(device, case):
    """The seeded corner-case batches of the stream decomposition (fewer blocks than wavefronts,
    empty requests, shares that begin on partition cuts, one long request among short ones) with
    the head dimension, the pool format and the block size drawn too."""
    from test_gpu_attn import _random_case
    rng = np.random.default_rng(31000 + case)
    lens, hq, hkv, P = _random_case(rng, case)
    D = int(rng.choice([64, 256]))
    fp8 = bool(rng.integers(0, 2))
    B = int(rng.choice([16, 32, 64]))
    if D == 256 and hq // hkv > 8:
        hq = 8 * hkv
    if P and P % B:
        P = B * (P // B + 1)
    need = int(((lens + B - 1) // B).sum())
    w = wl.custom(lens, hq, hkv, seed=3100 + case, partition_size=P, block_size=B, head_dim=D,
                  num_pool_blocks=need + int(rng.integers(1, 50)))
    what = f"case {case}: D={D} fp8={fp8} B={B} S={len(lens)} hq={hq} hkv={hkv} P={P} tokens={int(lens.sum())}"
    print(what, flush=True)
    if fp8:
        ks, vs = np.float32(0.0134), np.float32(0.0171)
        q, k, v = wl.make_host_tensors_fp8(w, ks, vs, poison_unused=True)
        assert_launchable(w)
        shape = shape_of(w)
        ws = torch.empty(max(pkv.pkv_attn_workspace_bytes(shape), 16), dtype=torch.uint8, device=device)
        out = torch.full(w.q_shape(), 0x7FC1, dtype=torch.int16, device=device)
        pkv.paged_decode_attn_fp8kv(to_dev(q), torch.from_numpy(k).to(device), torch.from_numpy(v).to(device),
                                    to_dev(w.block_tables), to_dev(w.context_lens), float(w.scale),
                                    float(ks), float(vs), out, shape, ws)
        torch.cuda.synchronize()
        got = to_bits(out)
        ref = oracle.paged_decode_attn_fp8kv(q, k, v, w.block_tables, w.context_lens, w.scale, ks, vs)
    else:
        q, k, v = wl.make_host_tensors(w, poison_unused=True)
        got = run_attn(w, q, k, v)
        ref = oracle.paged_decode_attn(q, k, v, w.block_tables, w.context_lens, w.scale)
    c = oracle.compare(got, ref)
    assert np.isfinite(wl.bf16_bits_to_f64(got)).all()
    assert c["rel_l2"] <= REL_L2 and c["worst_seq_rel_l2"] <= 2 * REL_L2, (what, c)
    assert abs_error_within_bar(got, ref), (what, c)
    for s in np.nonzero(lens == 0)[0]:
        assert not got.reshape(w.q_shape())[s].any()
