"""Preemption through the backing store: a request's KV blocks are offloaded to
pinned host memory and later reloaded into other blocks (paper Section II-B).
Bit-exact against the oracle's gather / scatter; attention after the round trip
is identical to attention before it."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_11530_amd import binding as pkv
from paper_2602_11530_amd import workloads as wl

from gpu_util import assert_launchable, run_attn_dev, to_bits, to_dev

pytestmark = pytest.mark.gpu


def pinned_like(n_blocks, block_shape):
    t = torch.empty((n_blocks,) + tuple(block_shape), dtype=torch.int16, pin_memory=True)
    assert t.is_pinned()
    t.fill_(0x5A5A)
    return t


def test_offload_and_reload_bit_exact(device):
    rng = np.random.default_rng(61)
    NB, blk = 97, (8, 16, 128)
    pool = rng.integers(0, 65536, size=(NB,) + blk).astype(np.uint16)
    ids = rng.permutation(NB)[:41].astype(np.int32)
    new_ids = rng.permutation(NB)[:41].astype(np.int32)
    bb = int(np.prod(blk)) * 2
    pool_d, ids_d, new_d = to_dev(pool), to_dev(ids), to_dev(new_ids)
    staging = torch.zeros((41,) + blk, dtype=torch.int16, device=device)
    host = pinned_like(41, blk)
    pkv.kv_blocks_offload(pool_d, ids_d, staging, host, 41, bb, NB)
    torch.cuda.synchronize()
    want = oracle.kv_blocks_gather(pool, ids)
    assert np.array_equal(host.numpy().view(np.uint16), want)
    assert np.array_equal(to_bits(pool_d), pool), "offload must not write the pool"
    # the freed blocks are reused by someone else, then the request comes back elsewhere
    pool_d[ids_d.long()] = 0x1111
    pool_now = to_bits(pool_d).copy()
    staging.fill_(0)
    pkv.kv_blocks_reload(host, staging, pool_d, new_d, 41, bb, NB)
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(pool_d), oracle.kv_blocks_scatter(want, pool_now, new_ids))
    # a pageable host buffer is refused before anything is enqueued
    pageable = torch.empty((41,) + blk, dtype=torch.int16)
    with pytest.raises(pkv.PkvError) as e:
        pkv.kv_blocks_offload(pool_d, ids_d, staging, pageable, 41, bb, NB)
    assert e.value.status == pkv.PKV_ERR_HOST
    with pytest.raises(pkv.PkvError) as e:
        pkv.kv_blocks_reload(staging, staging, pool_d, new_d, 41, bb, NB)   # device memory is not host memory
    assert e.value.status == pkv.PKV_ERR_HOST
    # empty list: nothing happens
    pkv.kv_blocks_offload(pool_d, ids_d, staging, host, 0, bb, NB)
    pkv.kv_blocks_reload(host, staging, pool_d, new_d, 0, bb, NB)


def test_preempt_then_resume_attention_unchanged(device):
    """Evict three requests of a batch, let their blocks be overwritten, resume
    them into different blocks: the batch's attention output is bit-identical to
    the one before the eviction."""
    w = wl.custom([900, 33, 2100, 16, 1500, 700], 40, 8, seed=63, num_pool_blocks=420)
    assert_launchable(w)
    q, k, v = wl.make_host_tensors(w)
    q_d, k_d, v_d = to_dev(q), to_dev(k), to_dev(v)
    t_d, l_d = to_dev(w.block_tables), to_dev(w.context_lens)
    before = run_attn_dev(w, q_d, k_d, v_d, t_d, l_d)
    ref = oracle.paged_decode_attn(q, k, v, w.block_tables, w.context_lens, w.scale)
    used = w.used_blocks()
    victims = [0, 2, 4]
    old = np.concatenate([w.block_tables[s, :int(used[s])] for s in victims]).astype(np.int32)
    in_use = np.concatenate([w.block_tables[s, :int(used[s])] for s in range(w.num_seqs)])
    free = np.setdiff1d(np.arange(w.num_pool_blocks), in_use)
    rng = np.random.default_rng(63)
    # come back into a mix of never-used blocks and the request's own old ones, reshuffled
    new = rng.permutation(np.concatenate([free, old]))[:len(old)].astype(np.int32)
    n, bb, NB = len(old), w.block_bytes, w.num_pool_blocks
    staging = torch.empty((n,) + tuple(w.pool_shape()[1:]), dtype=torch.int16, device=device)
    host_k, host_v = pinned_like(n, w.pool_shape()[1:]), pinned_like(n, w.pool_shape()[1:])
    old_d, new_d = to_dev(old), to_dev(new)
    pkv.kv_blocks_offload(k_d, old_d, staging, host_k, n, bb, NB)
    pkv.kv_blocks_offload(v_d, old_d, staging, host_v, n, bb, NB)
    torch.cuda.synchronize()
    k_d[old_d.long()] = 0x7FC1   # NaN patterns: anything still reading the old blocks would show
    v_d[old_d.long()] = 0x7FC1
    pkv.kv_blocks_reload(host_k, staging, k_d, new_d, n, bb, NB)
    pkv.kv_blocks_reload(host_v, staging, v_d, new_d, n, bb, NB)
    tables = w.block_tables.copy()
    off = 0
    for s in victims:
        tables[s, :int(used[s])] = new[off:off + int(used[s])]
        off += int(used[s])
    w_after = wl.Workload("resumed", w.num_q_heads, w.num_kv_heads, w.context_lens, tables,
                          w.num_pool_blocks, seed=w.seed)
    assert_launchable(w_after)
    after = run_attn_dev(w_after, q_d, k_d, v_d, to_dev(tables), l_d)
    torch.cuda.synchronize()
    assert torch.equal(before, after)
    c = oracle.compare(to_bits(after), ref)
    assert c["rel_l2"] <= 5e-3 and c["max_abs"] <= 1e-2, c


def test_offload_next_to_decode(device):
    """One layer of the phase-mixed batch: stream A evicts 25 % of the requests (K and
    V, about 0.39 GB each) to pinned memory and reloads them, stream B keeps decoding
    for the survivors.  Reports the PCIe-inclusive rates and what the concurrent
    copy costs the attention call."""
    w = wl.cfg4_phase_mixed(num_layers=1)
    mig = wl.make_migration(w, 0.25)
    g = torch.Generator(device=device)
    g.manual_seed(w.seed + 17)
    k_d = torch.randn(w.pool_shape(), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    v_d = torch.randn(w.pool_shape(), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    ws_surv = wl.subset(w, mig.survivors)
    assert_launchable(ws_surv)
    q_d = torch.randn(ws_surv.q_shape(), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    st_tables, st_lens = to_dev(ws_surv.block_tables), to_dev(ws_surv.context_lens)
    n, bb, NB = len(mig.old_ids), w.block_bytes, w.num_pool_blocks
    assert mig.old_ids.min() >= 0 and mig.old_ids.max() < NB and mig.new_ids.max() < NB
    old_d, new_d = to_dev(mig.old_ids), to_dev(mig.new_ids)
    staging = torch.empty((n,) + tuple(w.pool_shape()[1:]), dtype=torch.bfloat16, device=device)
    host_k, host_v = pinned_like(n, w.pool_shape()[1:]), pinned_like(n, w.pool_shape()[1:])
    want_k = k_d.index_select(0, old_d.long()).cpu()
    want_v = v_d.index_select(0, old_d.long()).cpu()
    stream_a, stream_b = torch.cuda.Stream(device), torch.cuda.Stream(device)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def evict():
        pkv.kv_blocks_offload(k_d, old_d, staging, host_k, n, bb, NB, stream_a)
        pkv.kv_blocks_offload(v_d, old_d, staging, host_v, n, bb, NB, stream_a)

    def resume():
        pkv.kv_blocks_reload(host_k, staging, k_d, new_d, n, bb, NB, stream_a)
        pkv.kv_blocks_reload(host_v, staging, v_d, new_d, n, bb, NB, stream_a)

    def timed_a(fn):
        a, b = ev(), ev()
        a.record(stream_a); fn(); b.record(stream_a)
        torch.cuda.synchronize()
        return a.elapsed_time(b)

    evict(); torch.cuda.synchronize()
    ms_out = timed_a(evict)
    assert torch.equal(host_k.view(torch.bfloat16), want_k) and torch.equal(host_v.view(torch.bfloat16), want_v)
    print(f"offload {2 * n * bb / 1e9:.2f} GB: {ms_out:.2f} ms = {2 * n * bb / ms_out / 1e6:.1f} GB/s "
          f"(gather + device-to-host copy)", flush=True)

    reps = 40
    from gpu_util import shape_of
    shape_s = shape_of(ws_surv)
    ws_b = torch.empty(pkv.pkv_attn_workspace_bytes(shape_s), dtype=torch.uint8, device=device)
    out = torch.full(ws_surv.q_shape(), 0x7FC1, dtype=torch.int16, device=device)
    torch.cuda.synchronize()   # the fill ran on the default stream; the side streams do not wait for it

    def decode(times):
        a, b = ev(), ev()
        a.record(stream_b)
        for _ in range(times):
            pkv.paged_decode_attn(q_d, k_d, v_d, st_tables, st_lens, float(w.scale), out, shape_s,
                                  ws_b, stream_b)
        b.record(stream_b)
        return a, b

    a, b = decode(reps); torch.cuda.synchronize()
    alone = out.clone()
    ms_alone = a.elapsed_time(b) / reps
    # both at once: the eviction is long enough to cover all the decode calls
    a0, b0 = ev(), ev()
    a0.record(stream_a); evict(); b0.record(stream_a)
    a, b = decode(reps)
    torch.cuda.synchronize()
    ms_both, ms_out_both = a.elapsed_time(b) / reps, a0.elapsed_time(b0)
    assert torch.equal(out, alone), "survivors' rows changed while the eviction ran"
    assert torch.equal(host_k.view(torch.bfloat16), want_k) and torch.equal(host_v.view(torch.bfloat16), want_v)
    print(f"attention for the 72 survivors: {ms_alone:.4f} ms alone, {ms_both:.4f} ms next to the offload "
          f"({ms_out_both:.2f} ms for the offload meanwhile)", flush=True)

    # survivors never touch the victims' old or new blocks, so the reload may overlap too
    k_d[old_d.long()] = 0
    v_d[old_d.long()] = 0
    torch.cuda.synchronize()   # default-stream writes before the reload on the side stream
    ms_in = timed_a(resume)
    assert torch.equal(k_d.index_select(0, new_d.long()).cpu(), want_k)
    assert torch.equal(v_d.index_select(0, new_d.long()).cpu(), want_v)
    print(f"reload  {2 * n * bb / 1e9:.2f} GB: {ms_in:.2f} ms = {2 * n * bb / ms_in / 1e6:.1f} GB/s "
          f"(host-to-device copy + scatter)", flush=True)
