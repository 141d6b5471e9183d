"""Physical blocks of 32 and 64 tokens: the kernels stream 16-token units, so a larger
block is two or four units in a row per KV head.  Same parity bar as for 16."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_11530_amd import binding as pkv
from paper_2602_11530_amd import workloads as wl

from gpu_util import (MAX_ABS, REL_L2, abs_error_within_bar, assert_launchable, run_attn, run_attn_dev,
                      shape_of, to_bits, to_dev)

pytestmark = pytest.mark.gpu

EDGE = [1, 15, 16, 17, 31, 32, 33, 47, 48, 49, 63, 64, 65, 0, 127, 128, 129, 511, 512, 513, 1000, 2]


def check(w, q, k, v, got, what, large_outputs_possible=False):
    ref = oracle.paged_decode_attn(q, k, v, w.block_tables, w.context_lens, w.scale)
    c = oracle.compare(got, ref)
    print(f"{what}: {c}", flush=True)
    assert np.isfinite(wl.bf16_bits_to_f64(got)).all()
    assert c["rel_l2"] <= REL_L2 and c["worst_seq_rel_l2"] <= 2 * REL_L2, c
    if large_outputs_possible:      # batches full of one- to three-token requests
        assert abs_error_within_bar(got, ref), c
    else:
        assert c["max_abs"] <= MAX_ABS, c


@pytest.mark.parametrize("B", [32, 64])
@pytest.mark.parametrize("hq,hkv", [(40, 8), (8, 2), (16, 1)])
@pytest.mark.parametrize("P", [0, 64, 512])
def test_edge_lengths(device, B, hq, hkv, P):
    w = wl.custom(EDGE, hq, hkv, seed=700 + B + hq, num_pool_blocks=300, partition_size=P, block_size=B)
    assert w.pool_shape()[2] == B
    q, k, v = wl.make_host_tensors(w, poison_unused=True)
    got = run_attn(w, q, k, v)
    check(w, q, k, v, got, f"B={B} hq={hq} hkv={hkv} P={P}")
    assert not got.reshape(w.q_shape())[EDGE.index(0)].any()


@pytest.mark.parametrize("B", [32, 64])
def test_block_size_does_not_change_the_result(device, B):
    """The same rows stored in blocks of 16 and in blocks of B give bit-identical output:
    the order of the arithmetic depends on token positions only."""
    lens = [1300, 77, 2048, 640, 33]
    w16 = wl.custom(lens, 40, 8, seed=81, block_size=16)
    wB = wl.custom(lens, 40, 8, seed=82, block_size=B)
    q, k16, v16 = wl.make_host_tensors(w16)
    kB = np.zeros(wB.pool_shape(), np.uint16)
    vB = np.zeros(wB.pool_shape(), np.uint16)
    for s, L in enumerate(lens):
        for t in range(L):
            src = (w16.block_tables[s, t // 16], slice(None), t % 16)
            dst = (wB.block_tables[s, t // B], slice(None), t % B)
            kB[dst], vB[dst] = k16[src], v16[src]
    a = run_attn(w16, q, k16, v16)
    b = run_attn(wB, q, kB, vB)
    assert np.array_equal(a, b)
    check(wB, q, kB, vB, b, f"B={B} re-blocked")


@pytest.mark.parametrize("B", [32, 64])
def test_append_then_attend(device, B):
    final = np.array([20, 2 * B, 2 * B + 1, 515, 1300, 3], np.int32)
    w = wl.custom(final, 40, 8, seed=90 + B, num_pool_blocks=80, block_size=B)
    rng = np.random.default_rng(B)
    q, k, v = wl.make_host_tensors(w)
    k_d, v_d, t_d = to_dev(k), to_dev(v), to_dev(w.block_tables)
    k_h, v_h = k.copy(), v.copy()
    for back in (2, 1, 0):
        w.context_lens = final - back
        assert_launchable(w)
        k_new = wl.normal_bf16(rng, (w.num_seqs, 8, 128))
        v_new = wl.normal_bf16(rng, (w.num_seqs, 8, 128))
        q = wl.normal_bf16(rng, w.q_shape())
        lens_d = to_dev(w.context_lens)
        pkv.kv_append(to_dev(k_new), to_dev(v_new), k_d, v_d, t_d, lens_d, shape_of(w))
        out = run_attn_dev(w, to_dev(q), k_d, v_d, t_d, lens_d)
        torch.cuda.synchronize()
        k_h, v_h = oracle.kv_append(k_new, v_new, k_h, v_h, w.block_tables, w.context_lens)
        assert np.array_equal(to_bits(k_d).reshape(k.shape), k_h)
        assert np.array_equal(to_bits(v_d).reshape(v.shape), v_h)
        check(w, q, k_h, v_h, to_bits(out), f"B={B} append step, lens {w.context_lens.tolist()}")


def test_cfg2_shape_with_blocks_of_64(device):
    """The headline batch stored in 64-token blocks: parity, and its time next to B = 16."""
    rng = np.random.default_rng(wl.BASE_SEED + 2)
    lens = rng.integers(1024, 8193, size=64).astype(np.int32)
    times = {}
    for B in (16, 64):
        w = wl.custom(lens, 40, 8, seed=wl.BASE_SEED + 2, block_size=B, maxb=8192 // B)
        g = torch.Generator(device=device); g.manual_seed(5)
        q = torch.randn(w.q_shape(), generator=g, device=device).to(torch.bfloat16)
        k = torch.randn(w.pool_shape(), generator=g, device=device).to(torch.bfloat16)
        v = torch.randn(w.pool_shape(), generator=g, device=device).to(torch.bfloat16)
        t_d, l_d = to_dev(w.block_tables), to_dev(w.context_lens)
        shape = shape_of(w)
        ws = torch.empty(pkv.pkv_attn_workspace_bytes(shape), dtype=torch.uint8, device=device)
        out = torch.full(w.q_shape(), 0x7FC1, dtype=torch.int16, device=device)
        run = lambda: pkv.paged_decode_attn(q, k, v, t_d, l_d, float(w.scale), out, shape, ws)
        for _ in range(5):
            run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(50):
            run()
        e1.record()
        torch.cuda.synchronize()
        times[B] = e0.elapsed_time(e1) / 50
        check(w, to_bits(q), to_bits(k), to_bits(v), to_bits(out), f"cfg2 lengths, B={B}")
        print(f"B={B}: {times[B]:.4f} ms, {w.attn_algorithmic_bytes() / times[B] / 1e6:.0f} GB/s", flush=True)


@pytest.mark.parametrize("case", range(48))
def test_random_shapes_all_block_sizes(device, case):
    """The seeded corner-case batches of the stream decomposition, with the block size drawn too
    (the partition size is raised to a multiple of it)."""
    from test_gpu_attn import _random_case
    rng = np.random.default_rng(12000 + case)
    lens, hq, hkv, P = _random_case(rng, case)
    B = int(rng.choice([16, 32, 64]))
    if P and P % B:
        P = B * (P // B + 1)
    need = int(((lens + B - 1) // B).sum())
    w = wl.custom(lens, hq, hkv, seed=1500 + case, partition_size=P, block_size=B,
                  num_pool_blocks=need + int(rng.integers(1, 50)))
    q, k, v = wl.make_host_tensors(w, poison_unused=True)
    got = run_attn(w, q, k, v)
    check(w, q, k, v, got, f"case {case}: B={B} S={len(lens)} hq={hq} hkv={hkv} P={P} tokens={int(lens.sum())}",
          large_outputs_possible=True)
    for s in np.nonzero(lens == 0)[0]:
        assert not got.reshape(w.q_shape())[s].any()
