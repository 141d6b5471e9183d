"""GPU parity of kv_blocks_gather / kv_blocks_scatter: bit-exact against the
checker's byte copies, and attention unchanged by a migration."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_11530_amd import binding as pkv
from paper_2602_11530_amd import workloads as wl

from gpu_util import run_attn, to_bits, to_dev

pytestmark = pytest.mark.gpu


def gather_gpu(pool_d, ids, block_bytes):
    nb = pool_d.shape[0]
    assert len(ids) == 0 or (0 <= min(ids) and max(ids) < nb)
    ids_d = to_dev(np.asarray(ids, np.int32))
    st = torch.full((len(ids) * block_bytes // 2,), 0x5A5A, dtype=torch.int16, device=pool_d.device)
    pkv.kv_blocks_gather(pool_d, ids_d, st, len(ids), block_bytes, nb)
    torch.cuda.synchronize()
    return st


@pytest.mark.parametrize("hkv,n", [(8, 37), (2, 5), (1, 1), (8, 1000)])
def test_gather_scatter_bit_exact(device, hkv, n):
    rng = np.random.default_rng(100 + n)
    NB = max(2 * n, 8)
    pool = rng.integers(0, 65536, size=(NB, hkv, 16, 128)).astype(np.uint16)
    bb = hkv * 16 * 128 * 2
    ids = rng.permutation(NB)[:n].astype(np.int32)
    pool_d = to_dev(pool)
    st = gather_gpu(pool_d, ids, bb)
    want = oracle.kv_blocks_gather(pool, ids)
    assert np.array_equal(to_bits(st).reshape(want.shape), want)
    assert np.array_equal(to_bits(pool_d), pool), "gather must not write the pool"

    new_ids = rng.permutation(NB)[:n].astype(np.int32)
    pkv.kv_blocks_scatter(st, pool_d, to_dev(new_ids), n, bb, NB)
    torch.cuda.synchronize()
    want_pool = oracle.kv_blocks_scatter(want, pool, new_ids)
    assert np.array_equal(to_bits(pool_d), want_pool)


def test_odd_block_bytes_and_empty_list(device):
    """block_bytes only has to be a multiple of 16; an empty list is a no-op."""
    rng = np.random.default_rng(7)
    for bb in (16, 48, 4096 + 16, 65536, 100000 - 100000 % 16):
        NB = 9
        pool = rng.integers(0, 65536, size=(NB, bb // 2)).astype(np.uint16)
        ids = np.array([8, 0, 3], np.int32)
        pool_d = to_dev(pool)
        st = gather_gpu(pool_d, ids, bb)
        assert np.array_equal(to_bits(st).reshape(3, -1), pool[ids])
        dst = to_dev(np.zeros_like(pool))
        pkv.kv_blocks_scatter(st, dst, to_dev(ids), 3, bb, NB)
        torch.cuda.synchronize()
        want = np.zeros_like(pool)
        want[ids] = pool[ids]
        assert np.array_equal(to_bits(dst), want)
    pkv.kv_blocks_gather(pool_d, to_dev(ids), st, 0, bb, NB)
    pkv.kv_blocks_scatter(st, pool_d, to_dev(ids), 0, bb, NB)
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(pool_d), pool)


def test_list_longer_than_the_grid(device):
    """More listed slices than the launch has workgroups (2^23): the kernel walks the list with a
    stride.  9 million blocks of 16 bytes, gathered, scattered and moved in a seeded order."""
    n = (1 << 23) + 600_001
    rng = np.random.default_rng(23)
    pool = rng.integers(0, 65536, size=(n, 8)).astype(np.uint16)
    ids = rng.permutation(n).astype(np.int32)
    pool_d = to_dev(pool)
    st = gather_gpu(pool_d, ids, 16)
    want = oracle.kv_blocks_gather(pool, ids)
    assert np.array_equal(to_bits(st).reshape(want.shape), want)
    new_ids = rng.permutation(n).astype(np.int32)
    dst = to_dev(np.zeros_like(pool))
    pkv.kv_blocks_scatter(st, dst, to_dev(new_ids), n, 16, n)
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(dst), oracle.kv_blocks_scatter(want, np.zeros_like(pool), new_ids))
    dst2 = to_dev(np.zeros_like(pool))
    pkv.kv_blocks_move(pool_d, to_dev(ids), dst2, to_dev(new_ids), n, 16, n, n)
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(dst2), to_bits(dst))


def test_migration_keeps_attention_bitwise(device):
    """Gather a quarter of the requests, scatter into reshuffled blocks, rewrite
    their tables: every block image and the attention output are unchanged."""
    w = wl.custom([300, 1000, 77, 513, 16, 2000, 40, 900], 40, 8, seed=21, num_pool_blocks=400)
    q, k, v = wl.make_host_tensors(w)
    before = run_attn(w, q, k, v)
    mig = wl.make_migration(w, 0.25)
    pools = []
    for pool in (k, v):
        pool_d = to_dev(pool)
        st = gather_gpu(pool_d, mig.old_ids, w.block_bytes)
        pkv.kv_blocks_scatter(st, pool_d, to_dev(mig.new_ids), len(mig.new_ids), w.block_bytes,
                              w.num_pool_blocks)
        torch.cuda.synchronize()
        got = to_bits(pool_d).reshape(pool.shape)
        want = oracle.kv_blocks_scatter(oracle.kv_blocks_gather(pool, mig.old_ids), pool, mig.new_ids)
        assert np.array_equal(got, want)
        assert np.array_equal(got[mig.new_ids], pool[mig.old_ids])
        pools.append(got)
    w2 = wl.Workload("after", 40, 8, w.context_lens, mig.tables_after, w.num_pool_blocks, seed=w.seed)
    after = run_attn(w2, q, pools[0], pools[1])
    assert np.array_equal(before, after)


@pytest.mark.expects_id_faults
def test_out_of_range_ids_are_skipped(device, id_faults):
    """The device never follows an id outside the pool: those list entries are
    skipped, reported through the fault counter, and everything else is copied
    as usual."""
    rng = np.random.default_rng(9)
    NB, bb = 12, 8 * 16 * 128 * 2
    pool = rng.integers(0, 65536, size=(NB, bb // 2)).astype(np.uint16)
    ids = np.array([3, -1, 11, NB, 0, 2 ** 31 - 1, -2 ** 31], np.int32)
    ok = (ids >= 0) & (ids < NB)
    pool_d = to_dev(pool)
    st = torch.full((len(ids) * bb // 2,), 0x5A5A, dtype=torch.int16, device=pool_d.device)
    pkv.kv_blocks_gather(pool_d, to_dev(ids), st, len(ids), bb, NB)
    torch.cuda.synchronize()
    got = to_bits(st).reshape(len(ids), -1)
    assert np.array_equal(got[ok], pool[ids[ok]]) and (got[~ok] == 0x5A5A).all()
    assert int(id_faults.item()) == int((~ok).sum())
    dst = to_dev(np.zeros_like(pool))
    pkv.kv_blocks_scatter(st, dst, to_dev(ids), len(ids), bb, NB)
    torch.cuda.synchronize()
    assert int(id_faults.item()) == 2 * int((~ok).sum())
    # pool to pool: an entry is skipped, and counted once, when either of its ids is out of range
    other = to_dev(np.zeros_like(pool))
    good_ids = np.arange(len(ids), dtype=np.int32)
    pkv.kv_blocks_move(pool_d, to_dev(ids), other, to_dev(good_ids), len(ids), bb, NB, NB)
    pkv.kv_blocks_move(pool_d, to_dev(good_ids), other, to_dev(ids), len(ids), bb, NB, NB)
    torch.cuda.synchronize()
    assert int(id_faults.item()) == 4 * int((~ok).sum())
    # switched off: nothing is counted, the entries are still skipped
    pkv.pkv_set_id_fault_counter(None)
    pkv.kv_blocks_gather(pool_d, to_dev(ids), st, len(ids), bb, NB)
    torch.cuda.synchronize()
    assert int(id_faults.item()) == 4 * int((~ok).sum())
    pkv.pkv_set_id_fault_counter(id_faults)
    want = np.zeros_like(pool)
    want[ids[ok]] = pool[ids[ok]]
    assert np.array_equal(to_bits(dst), want)


@pytest.mark.expects_id_faults
@pytest.mark.parametrize("hkv,n", [(8, 37), (2, 5), (1, 1), (8, 700)])
def test_move_bit_exact(device, hkv, n, id_faults):
    """Pool to pool in one pass equals the oracle's move, and gather + scatter."""
    rng = np.random.default_rng(300 + n)
    NBs, NBd = max(2 * n, 8), max(3 * n, 5)
    src = rng.integers(0, 65536, size=(NBs, hkv, 16, 128)).astype(np.uint16)
    dst = rng.integers(0, 65536, size=(NBd, hkv, 16, 128)).astype(np.uint16)
    bb = hkv * 16 * 128 * 2
    a = rng.permutation(NBs)[:n].astype(np.int32)
    b = rng.permutation(NBd)[:n].astype(np.int32)
    src_d, dst_d = to_dev(src), to_dev(dst)
    pkv.kv_blocks_move(src_d, to_dev(a), dst_d, to_dev(b), n, bb, NBs, NBd)
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(dst_d), oracle.kv_blocks_move(src, a, dst, b))
    assert np.array_equal(to_bits(src_d), src), "the source pool must not change"
    assert int(id_faults.item()) == 0
    # out-of-range entries on either side are skipped, the rest still moves
    a2, b2 = a.copy(), b.copy()
    a2[0] = NBs + 3
    if n > 1:
        b2[-1] = -1
    dst_d = to_dev(dst)
    pkv.kv_blocks_move(src_d, to_dev(a2), dst_d, to_dev(b2), n, bb, NBs, NBd)
    torch.cuda.synchronize()
    keep = np.ones(n, bool)
    keep[0] = False
    if n > 1:
        keep[-1] = False
    assert int(id_faults.item()) == int((~keep).sum())
    assert np.array_equal(to_bits(dst_d), oracle.kv_blocks_move(src, a[keep], dst, b[keep]))


def test_move_within_one_pool_and_timing(device):
    """Disjoint source and destination blocks of the same pool (cfg5's size: the KV of 24 of
    96 requests, one layer's K pool); time against gather + scatter through staging."""
    w = wl.cfg4_phase_mixed(num_layers=1)
    mig = wl.make_migration(w, 0.25)
    n, bb = len(mig.old_ids), w.block_bytes
    NB = w.num_pool_blocks + n                      # the batch's blocks plus as many spare ones
    rng = np.random.default_rng(5)
    old = mig.old_ids.astype(np.int32)
    new = (w.num_pool_blocks + rng.permutation(n)).astype(np.int32)
    g = torch.Generator(device=device); g.manual_seed(3)
    pool = torch.randint(-32768, 32767, (NB,) + tuple(w.pool_shape()[1:]), generator=g, device=device,
                         dtype=torch.int16)
    before = pool.clone()
    old_d, new_d = to_dev(old), to_dev(new)
    staging = torch.empty((n,) + tuple(w.pool_shape()[1:]), dtype=torch.int16, device=device)

    def timed(fn, reps=20):
        fn(); torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    ms_move = timed(lambda: pkv.kv_blocks_move(pool, old_d, pool, new_d, n, bb, NB, NB))
    assert torch.equal(pool.index_select(0, new_d.long()), before.index_select(0, old_d.long()))
    untouched = torch.from_numpy(np.setdiff1d(np.arange(NB), new)).to(device)
    assert torch.equal(pool.index_select(0, untouched), before.index_select(0, untouched))

    def two_step():
        pkv.kv_blocks_gather(pool, old_d, staging, n, bb, NB)
        pkv.kv_blocks_scatter(staging, pool, new_d, n, bb, NB)
    ms_two = timed(two_step)
    print(f"{n} blocks ({n * bb / 1e6:.0f} MB): move {ms_move * 1e3:.1f} us = {2 * n * bb / ms_move / 1e6:.0f} GB/s "
          f"read+write; gather + scatter {ms_two * 1e3:.1f} us", flush=True)
    assert ms_move < ms_two
