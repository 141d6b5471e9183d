"""Pools larger than 4 GiB: every byte offset the kernels form from a block id must be a 64-bit
one.  The pools are 150 000 blocks of 32 KiB (4.9 GB each); the requests' blocks are spread over
the whole pool, one sits on the pool's last block and one just past the 4 GiB mark.  Only the
blocks in use carry data (the rest is zero and never read), so the host copies stay small."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_11530_amd import binding as pkv
from paper_2602_11530_amd import workloads as wl

from gpu_util import MAX_ABS, REL_L2, run_attn_dev, shape_of, to_bits, to_dev

pytestmark = pytest.mark.gpu

NB = 150_000


def sparse_pools(w, rng, device):
    """Host pool (zero pages except the used blocks) and its device twin."""
    ids = np.unique(w.block_tables[w.block_tables >= 0])
    pools = []
    for _ in range(2):
        host = np.zeros(w.pool_shape(), dtype=np.uint16)          # untouched pages stay unmapped
        host[ids] = wl.normal_bf16(rng, (len(ids),) + w.pool_shape()[1:])
        dev = torch.zeros(w.pool_shape(), dtype=torch.int16, device=device)
        dev[to_dev(ids.astype(np.int64))] = to_dev(host[ids])
        pools.append((host, dev))
    return ids, pools


def test_attention_append_and_copies_beyond_4_gib(device):
    free, _ = torch.cuda.mem_get_info()
    if free < 14 * (1 << 30):
        pytest.skip("needs 14 GiB of free device memory")
    w = wl.custom([3000, 33, 6000, 16, 1], 40, 8, seed=4242, num_pool_blocks=NB)
    past_4g = (1 << 32) // w.block_bytes + 1
    w.block_tables[0, 0] = NB - 1            # the pool's last block
    w.block_tables[2, 5] = past_4g           # first block that begins beyond 4 GiB
    w.block_tables[4, 0] = NB - 2            # a one-token request near the end
    assert w.num_pool_blocks * w.block_bytes > (1 << 32)
    rng = np.random.default_rng(4242)
    ids, ((k_h, k_d), (v_h, v_d)) = sparse_pools(w, rng, device)
    assert (ids.astype(np.int64) * w.block_bytes > (1 << 32)).sum() >= 40
    q = wl.normal_bf16(rng, w.q_shape())
    t_d, l_d = to_dev(w.block_tables), to_dev(w.context_lens)

    # the new token's rows go into the last slot of every request, then attention
    S, Hkv, D = w.num_seqs, w.num_kv_heads, w.head_dim
    k_new, v_new = wl.normal_bf16(rng, (S, Hkv, D)), wl.normal_bf16(rng, (S, Hkv, D))
    pkv.kv_append(to_dev(k_new), to_dev(v_new), k_d, v_d, t_d, l_d, shape_of(w))
    k_h, v_h = oracle.kv_append(k_new, v_new, k_h, v_h, w.block_tables, w.context_lens)
    got = to_bits(run_attn_dev(w, to_dev(q), k_d, v_d, t_d, l_d))
    torch.cuda.synchronize()
    ids_d = to_dev(ids.astype(np.int64))
    assert np.array_equal(to_bits(k_d[ids_d]), k_h[ids]) and np.array_equal(to_bits(v_d[ids_d]), v_h[ids])
    ref = oracle.paged_decode_attn(q, k_h, v_h, w.block_tables, w.context_lens, w.scale)
    c = oracle.compare(got, ref)
    print(f"pools of {NB * w.block_bytes / 2**30:.2f} GiB: {c}", flush=True)
    assert c["max_abs"] <= MAX_ABS and c["rel_l2"] <= REL_L2 and c["worst_seq_rel_l2"] <= 2 * REL_L2, c
    # one token in the second-to-last block: the row is that V row, bit for bit
    assert np.array_equal(got.reshape(w.q_shape())[4].reshape(Hkv, 5, D),
                          np.repeat(v_h[NB - 2, :, 0, :][:, None, :], 5, axis=1))

    # gather blocks from both sides of the 4 GiB mark, scatter them to unused ids on both sides
    src = np.array([NB - 1, past_4g, int(ids[0]), int(ids[len(ids) // 2])], np.int32)
    unused = np.setdiff1d(np.array([NB - 3, past_4g + 7, 11, past_4g - 2], np.int32), ids)
    assert len(unused) == 4
    dst = unused.astype(np.int32)
    n, bb = len(src), w.block_bytes
    staging = torch.zeros((n,) + w.pool_shape()[1:], dtype=torch.int16, device=device)
    pkv.kv_blocks_gather(k_d, to_dev(src), staging, n, bb, NB)
    pkv.kv_blocks_scatter(staging, k_d, to_dev(dst), n, bb, NB)
    pkv.kv_blocks_move(v_d, to_dev(src), v_d, to_dev(dst), n, bb, NB, NB)
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(staging), oracle.kv_blocks_gather(k_h, src))
    dst_d = to_dev(dst.astype(np.int64))
    assert np.array_equal(to_bits(k_d[dst_d]), k_h[src])
    assert np.array_equal(to_bits(v_d[dst_d]), v_h[src])
    # nothing else moved: the used blocks still hold what they held
    assert np.array_equal(to_bits(k_d[ids_d]), k_h[ids]) and np.array_equal(to_bits(v_d[ids_d]), v_h[ids])
