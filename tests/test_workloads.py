"""The seeded generators produce the shapes and length mixes the configs name."""
import numpy as np

from paper_2602_11530_amd import workloads as wl


def _tables_ok(w):
    used = w.used_blocks()
    seen = []
    for s in range(w.num_seqs):
        row = w.block_tables[s]
        n = int(used[s])
        assert (row[:n] >= 0).all() and (row[:n] < w.num_pool_blocks).all()
        assert (row[n:] == -1).all()
        seen.append(row[:n])
    allb = np.concatenate(seen)
    assert len(np.unique(allb)) == len(allb), "a physical block is mapped twice"


def test_cfg1():
    w = wl.cfg1_tiny()
    assert (w.num_seqs, w.num_q_heads, w.num_kv_heads, w.num_pool_blocks) == (4, 8, 2, 128)
    assert w.max_blocks_per_seq == 19 and abs(float(w.scale) - 128 ** -0.5) < 1e-8
    _tables_ok(w)
    w2 = wl.cfg1_tiny()
    assert np.array_equal(w.block_tables, w2.block_tables)


def test_cfg2_pool_fits_exactly():
    w = wl.cfg2_qwen32b()
    assert (w.num_seqs, w.num_q_heads, w.num_kv_heads) == (64, 40, 8)
    assert w.context_lens.min() >= 1024 and w.context_lens.max() <= 8192
    assert w.num_pool_blocks == int(w.used_blocks().sum()) and w.max_blocks_per_seq == 512
    _tables_ok(w)
    kv = 2 * w.total_tokens * 8 * 128 * 2
    assert 0.9e9 < kv < 1.5e9
    assert kv < w.attn_algorithmic_bytes() < kv * 1.01


def test_cfg3_lognormal():
    w = wl.cfg3_long_cot()
    assert w.num_seqs == 128 and w.partition_size == 512 and w.max_blocks_per_seq == 2048
    assert w.context_lens.min() >= 512 and w.context_lens.max() <= 32768
    assert 4000 < np.median(w.context_lens) < 8500
    _tables_ok(w)


def test_cfg4_mix_and_cfg5_migration():
    w = wl.cfg4_phase_mixed()
    assert w.num_seqs == 96 and w.num_layers == 64 and int(w.phase.sum()) == 67
    r, a = w.context_lens[w.phase == 1], w.context_lens[w.phase == 0]
    assert r.min() >= 4096 and r.max() <= 16384 and a.min() >= 1024 and a.max() <= 4096
    _tables_ok(w)
    resident = 64 * 2 * w.num_pool_blocks * w.block_bytes
    assert 150e9 < resident < 240e9
    mig = wl.make_migration(w, 0.25)
    assert len(mig.victims) == 24 and len(mig.survivors) == 72
    assert len(np.unique(mig.new_ids)) == len(mig.new_ids) == len(mig.old_ids)
    used = w.used_blocks()
    surv = np.concatenate([w.block_tables[s, :int(used[s])] for s in mig.survivors])
    assert len(np.intersect1d(surv, mig.new_ids)) == 0, "scatter would hit a survivor's block"
    assert len(np.intersect1d(surv, mig.old_ids)) == 0
    w_after = wl.Workload("after", 40, 8, w.context_lens, mig.tables_after, w.num_pool_blocks)
    _tables_ok(w_after)


def test_poison_only_hits_unreadable_slots():
    w = wl.cfg1_tiny()
    q, k, v = wl.make_host_tensors(w)
    qp, kp, vp = wl.make_host_tensors(w, poison_unused=True)
    assert np.array_equal(q, qp)
    for s in range(w.num_seqs):
        L = int(w.context_lens[s])
        for t in range(L):
            pb = w.block_tables[s, t // 16]
            assert np.array_equal(k[pb, :, t % 16], kp[pb, :, t % 16])
            assert np.array_equal(v[pb, :, t % 16], vp[pb, :, t % 16])
    assert (kp == wl.BF16_NAN).sum() > 0 and (vp == wl.BF16_INF).sum() > 0
