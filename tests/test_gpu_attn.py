"""GPU parity of paged_decode_attn (through the C ABI) against the fp64 checker.

Bar: max-abs <= 1e-2 and relative L2 <= 5e-3 over each call's whole output
(bf16 in/out, fp32 accumulate)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_11530_amd import workloads as wl

from gpu_util import MAX_ABS, REL_L2, device_tensors, run_attn, run_attn_dev, to_bits, to_dev

pytestmark = pytest.mark.gpu


def check(w, q, k, v, got, what=""):
    ref = oracle.paged_decode_attn(q, k, v, w.block_tables, w.context_lens, w.scale)
    c = oracle.compare(got, ref)
    print(f"{w.name} {what}: {c}", flush=True)
    assert np.isfinite(wl.bf16_bits_to_f64(got)).all(), "non-finite output"
    assert c["max_abs"] <= MAX_ABS and c["rel_l2"] <= REL_L2, c
    # no single short request may hide in the batch
    assert c["worst_seq_rel_l2"] <= 2 * REL_L2, c
    return ref


@pytest.mark.parametrize("poison", [False, True])
def test_cfg1_tiny(device, poison):
    w = wl.cfg1_tiny()
    q, k, v = wl.make_host_tensors(w, poison_unused=poison)
    check(w, q, k, v, run_attn(w, q, k, v), f"poison={poison}")


EDGE = [1, 15, 16, 17, 31, 32, 33, 0, 255, 256, 257, 511, 512, 513, 2, 1000]


@pytest.mark.parametrize("hq,hkv", [(8, 2), (40, 8), (5, 1), (8, 8), (6, 2), (16, 2), (16, 1), (12, 1),
                                    (9, 3)])
@pytest.mark.parametrize("P", [0, 16, 512])
def test_edge_lengths(device, hq, hkv, P):
    w = wl.custom(EDGE, hq, hkv, seed=31 + hq, num_pool_blocks=400, partition_size=P)
    q, k, v = wl.make_host_tensors(w, poison_unused=True)
    got = run_attn(w, q, k, v)
    check(w, q, k, v, got, f"hq={hq} hkv={hkv} P={P}")
    zero_rows = got.reshape(w.q_shape())[EDGE.index(0)]
    assert not zero_rows.any(), "an empty request must get an all-zero row"


def test_quantum_and_demotion_lengths(device):
    """Lengths around the scheduler's token quantum (500) and demotion threshold
    (5000 tokens) of the paper's evaluation set-up (Section V-A)."""
    w = wl.custom([499, 500, 501, 4999, 5000, 5001], 40, 8, seed=77, partition_size=512)
    q, k, v = wl.make_host_tensors(w, poison_unused=True)
    check(w, q, k, v, run_attn(w, q, k, v))


def test_partition_size_invariance(device):
    w = wl.custom([1300, 700, 45, 2048], 40, 8, seed=5)
    q, k, v = wl.make_host_tensors(w)
    outs = {}
    for P in (16, 128, 512, 4096, 0):
        outs[P] = run_attn(w, q, k, v, partition_size=P)
        check(w, q, k, v, outs[P], f"P={P}")
    a = wl.bf16_bits_to_f64(outs[16])
    for P, o in outs.items():
        d = wl.bf16_bits_to_f64(o) - a
        assert np.sqrt((d * d).sum() / (a * a).sum()) <= REL_L2


def test_max_context_len_hint_only_shrinks_launch(device):
    w = wl.custom([300, 90, 17], 8, 2, seed=8, maxb=64, partition_size=64)
    q, k, v = wl.make_host_tensors(w)
    full = run_attn(w, q, k, v)
    hinted = run_attn(w, q, k, v, max_context_len=304)
    assert np.array_equal(full, hinted)


def test_length_one_is_v_bit_exact(device):
    """A one-token context returns its V row bit for bit — subnormals, the smallest normals and the
    largest finite values included (request 3 holds them); the one exception is a negative zero,
    which comes out as +0 (the accumulator starts at +0)."""
    w = wl.custom([1, 1, 1, 1], 40, 8, seed=3, num_pool_blocks=64)
    q, k, v = wl.make_host_tensors(w, poison_unused=True)
    corners = np.array([0x0001, 0x0040, 0x007F, 0x0080, 0x0081, 0x8001, 0x807F, 0x8080, 0x0000, 0x8000,
                        0x7F7F, 0xFF7F, 0x0100, 0x3F80, 0x0002, 0x0010] * 8, np.uint16)
    v[w.block_tables[3, 0], :, 0, :] = corners
    got = run_attn(w, q, k, v).reshape(w.q_shape())
    for s in range(4):
        for h in range(40):
            want = v[w.block_tables[s, 0], h // 5, 0].copy()
            want[want == 0x8000] = 0
            assert np.array_equal(got[s, h], want)


def test_v_ones_gives_exact_ones(device):
    """The softmax weights sum to one."""
    w = wl.custom([700, 33, 16, 1234], 40, 8, seed=4)
    q, k, v = wl.make_host_tensors(w)
    v[:] = 0x3F80
    for P in (0, 128):
        got = run_attn(w, q, k, v, partition_size=P)
        assert (got == 0x3F80).all()


def test_scale_zero_is_mean(device):
    w = wl.custom([37, 16, 100, 600], 8, 2, seed=9, num_pool_blocks=80)
    q, k, v = wl.make_host_tensors(w, poison_unused=True)
    got = run_attn(w, q, k, v, scale=0.0)
    ref = oracle.paged_decode_attn(q, k, v, w.block_tables, w.context_lens, 0.0)
    c = oracle.compare(got, ref)
    assert c["max_abs"] <= MAX_ABS and c["rel_l2"] <= REL_L2, c


def test_paging_invariance_bitwise(device):
    """Moving rows to other physical blocks (tables rewritten) changes nothing:
    the reduction order depends on logical positions only."""
    w = wl.custom([300, 1000, 77], 40, 8, seed=12, num_pool_blocks=200)
    q, k, v = wl.make_host_tensors(w)
    a = run_attn(w, q, k, v)
    perm = np.random.default_rng(1).permutation(w.num_pool_blocks)
    k2, v2 = np.empty_like(k), np.empty_like(v)
    k2[perm], v2[perm] = k, v
    w2 = wl.Workload("perm", 40, 8, w.context_lens,
                     np.where(w.block_tables >= 0, perm[np.clip(w.block_tables, 0, None)],
                              -1).astype(np.int32), w.num_pool_blocks, seed=w.seed)
    b = run_attn(w2, q, k2, v2)
    assert np.array_equal(a, b)


def test_batch_independence(device):
    """Continuous batching: dropping or reordering requests leaves the others'
    rows unchanged up to where their partial sums are split (which follows the
    lengths ahead of them in the batch)."""
    w = wl.custom([300, 1000, 77, 513, 16], 40, 8, seed=13)
    q, k, v = wl.make_host_tensors(w)
    a = run_attn(w, q, k, v).reshape(w.q_shape())
    ref = check(w, q, k, v, a)
    idx = [3, 0, 4]
    sub = wl.subset(w, idx)
    b = run_attn(sub, q[idx], k, v).reshape(sub.q_shape())
    c = oracle.compare(b, ref[idx])
    assert c["max_abs"] <= MAX_ABS and c["rel_l2"] <= REL_L2, c
    d = wl.bf16_bits_to_f64(b) - wl.bf16_bits_to_f64(a[idx])
    assert np.abs(d).max() <= 2.0 ** -7 * np.abs(wl.bf16_bits_to_f64(a)).max()   # a bf16 ulp or so
    # a batch repeated with the same lengths is bit-reproducible
    assert np.array_equal(run_attn(w, q, k, v).reshape(w.q_shape()), a)


def test_gqa_equals_mha_with_repeated_kv(device):
    w = wl.custom([300, 77, 600], 8, 2, seed=14)
    q, k, v = wl.make_host_tensors(w)
    a = run_attn(w, q, k, v)
    w_mha = wl.Workload("mha", 8, 8, w.context_lens, w.block_tables, w.num_pool_blocks, seed=w.seed)
    b = run_attn(w_mha, q, np.repeat(k, 4, axis=1), np.repeat(v, 4, axis=1))
    ref = check(w, q, k, v, a, "gqa")
    cb = oracle.compare(b, ref)
    assert cb["rel_l2"] <= REL_L2 and cb["max_abs"] <= MAX_ABS


def test_shared_prefix_blocks(device):
    """Several requests may map the same physical blocks (read-only sharing)."""
    w = wl.custom([200, 200, 90], 8, 2, seed=15, num_pool_blocks=64)
    w.block_tables[1, :5] = w.block_tables[0, :5]
    q, k, v = wl.make_host_tensors(w)
    check(w, q, k, v, run_attn(w, q, k, v))


def test_grow_by_one_token(device):
    """A request's cache grows by one row per decode step (paper Section II-A)."""
    final = np.array([50, 515], np.int32)
    w = wl.custom(final, 8, 2, seed=16, num_pool_blocks=64, maxb=40)   # tables cover the final lengths
    q, k, v = wl.make_host_tensors(w)
    for back in (3, 2, 1, 0):
        w.context_lens = final - back      # the slots ahead already hold N(0,1) rows
        assert (w.used_blocks() <= (w.block_tables >= 0).sum(1)).all()
        check(w, q, k, v, run_attn(w, q, k, v), f"lens={w.context_lens.tolist()}")


def test_cfg2_full_parity(device):
    w = wl.cfg2_qwen32b()
    q_d, k_d, v_d = device_tensors(w)
    out = run_attn_dev(w, q_d, k_d, v_d, to_dev(w.block_tables), to_dev(w.context_lens))
    torch.cuda.synchronize()
    check(w, to_bits(q_d), to_bits(k_d), to_bits(v_d), to_bits(out))


def test_cfg3_full_parity(device):
    w = wl.cfg3_long_cot()
    q_d, k_d, v_d = device_tensors(w)
    out = run_attn_dev(w, q_d, k_d, v_d, to_dev(w.block_tables), to_dev(w.context_lens))
    torch.cuda.synchronize()
    got = to_bits(out)
    q, k, v = to_bits(q_d), to_bits(k_d), to_bits(v_d)
    del k_d, v_d
    check(w, q, k, v, got)


@pytest.mark.expects_id_faults
def test_corrupt_table_entries_are_not_followed(device, id_faults):
    """Ids outside the pool are never dereferenced: the tokens of such a block
    drop out of the softmax, the other requests' rows are untouched, and the
    refused entries are reported through the fault counter."""
    w = wl.custom([300, 1000, 77, 40], 40, 8, seed=19, num_pool_blocks=200, partition_size=128)
    q, k, v = wl.make_host_tensors(w)
    good = run_attn(w, q, k, v).reshape(w.q_shape())
    assert int(id_faults.item()) == 0
    bad = wl.Workload("bad", 40, 8, w.context_lens, w.block_tables.copy(), w.num_pool_blocks,
                      partition_size=128, seed=w.seed)
    bad.block_tables[0, 3] = -7
    bad.block_tables[1, 10] = w.num_pool_blocks
    bad.block_tables[1, 11] = 2 ** 31 - 1
    bad.block_tables[3, :3] = -1            # nothing of request 3 is mapped
    dev = [to_dev(x) for x in (q, k, v, bad.block_tables, bad.context_lens)]
    out = run_attn_dev(bad, *dev, check_tables=False)
    torch.cuda.synchronize()
    got = to_bits(out).reshape(w.q_shape())
    # one report per refused 16-token unit and KV head: 1 + 2 + 3 table entries x 8 heads
    assert int(id_faults.item()) == (1 + 2 + 3) * 8
    assert np.array_equal(got[2], good[2])
    assert not got[3].any()
    # requests 0 and 1 equal the checker's result with the unmapped tokens removed
    keep = wl.custom([300 - 16, 1000 - 32], 40, 8, seed=1, num_pool_blocks=200)
    keep.block_tables[0, :18] = np.delete(w.block_tables[0, :19], 3)
    keep.block_tables[1, :61] = np.delete(w.block_tables[1, :63], [10, 11])
    ref = oracle.paged_decode_attn(q[:2], k, v, keep.block_tables, keep.context_lens, w.scale)
    c = oracle.compare(got[:2], ref)
    assert c["max_abs"] <= MAX_ABS and c["rel_l2"] <= REL_L2, c


def test_bench_launch_configuration(device):
    """Config 2 exactly as bench.py launches it: library-chosen partitioning and
    the batch's true maximum length as the host bound."""
    w = wl.cfg2_qwen32b()
    q_d, k_d, v_d = device_tensors(w)
    out = run_attn_dev(w, q_d, k_d, v_d, to_dev(w.block_tables), to_dev(w.context_lens),
                       partition_size=0, max_context_len=int(w.context_lens.max()))
    torch.cuda.synchronize()
    check(w, to_bits(q_d), to_bits(k_d), to_bits(v_d), to_bits(out), "bench configuration")


def _random_case(rng, case):
    hkv = int(rng.choice([1, 2, 4, 8]))
    g = int(rng.choice([1, 2, 4, 5, 7, 8, 16]))
    kind = case % 6
    if kind == 0:      # a handful of blocks: fewer blocks than persistent wavefronts
        lens = rng.integers(0, 40, size=int(rng.integers(1, 6)))
    elif kind == 1:    # many short requests, some empty
        lens = rng.integers(0, 100, size=int(rng.integers(50, 300)))
        lens[rng.random(len(lens)) < 0.2] = 0
    elif kind == 2:    # block count right around the number of wavefronts
        n = max(1, 2048 // hkv)
        lens = np.full(int(rng.integers(1, 4)), 16 * (n // 2), dtype=np.int64)
        lens[0] += int(rng.integers(-40, 40))
    elif kind == 3:    # lengths on exact partition multiples: shares start on partition cuts
        lens = 512 * rng.integers(1, 9, size=int(rng.integers(2, 20)))
    elif kind == 4:    # one long request among short ones
        lens = np.concatenate([rng.integers(1, 64, size=20), [int(rng.integers(5000, 20000))]])
    else:              # mixed
        lens = rng.integers(1, 3000, size=int(rng.integers(1, 40)))
    P = int(rng.choice([0, 16, 32, 64, 256, 512, 1024, 2048]))
    return np.maximum(np.asarray(lens, dtype=np.int64), 0), hkv * g, hkv, P


@pytest.mark.parametrize("case", range(36))
def test_random_shapes(device, case):
    """Seeded random batches aimed at the corners of the stream decomposition:
    fewer blocks than wavefronts, shares that begin on partition boundaries, empty
    requests, every group size."""
    rng = np.random.default_rng(9000 + case)
    lens, hq, hkv, P = _random_case(rng, case)
    w = wl.custom(lens, hq, hkv, seed=500 + case, partition_size=P,
                  num_pool_blocks=int(((lens + 15) // 16).sum()) + int(rng.integers(1, 50)))
    q, k, v = wl.make_host_tensors(w, poison_unused=True)
    got = run_attn(w, q, k, v)
    check(w, q, k, v, got, f"case {case}: S={len(lens)} hq={hq} hkv={hkv} P={P} tokens={int(lens.sum())}")
    for s in np.nonzero(lens == 0)[0]:
        assert not got.reshape(w.q_shape())[s].any()


@pytest.mark.parametrize("hq,hkv", [(8, 2), (16, 1)])
def test_maximum_batch(device, hq, hkv):
    """2048 requests in one call (the most the library takes): the per-request prefix arrays
    fill the LDS budget and leave room for a single parked record at G = 16."""
    rng = np.random.default_rng(77 + hq)
    lens = rng.integers(0, 120, size=2048)
    lens[[0, 5, 2047]] = [0, 1, 119]
    w = wl.custom(lens, hq, hkv, seed=880 + hq, partition_size=int(rng.choice([0, 32])))
    q, k, v = wl.make_host_tensors(w, poison_unused=True)
    got = run_attn(w, q, k, v)
    check(w, q, k, v, got, f"S=2048 hq={hq} hkv={hkv}")
    for s in np.nonzero(lens == 0)[0][:5]:
        assert not got.reshape(w.q_shape())[s].any()


def test_one_very_long_request(device):
    """131 072 tokens in one request (two partitions of the largest size), next to short ones."""
    w = wl.custom([131072, 3, 700], 8, 1, seed=991)
    q, k, v = wl.make_host_tensors(w)
    check(w, q, k, v, run_attn(w, q, k, v), "L=131072")


def test_length_bound_clamps_and_negative_length_is_empty(device):
    """A request longer than max_context_len is attended up to the bound; a negative length
    counts as zero.  Both are what the header promises for inputs a scheduler should not send."""
    w = wl.custom([300, 90, 17, 40], 8, 2, seed=18, maxb=32)
    q, k, v = wl.make_host_tensors(w)
    lens = w.context_lens.copy()
    lens[3] = -5
    q_d, k_d, v_d = (to_dev(x) for x in (q, k, v))
    got = to_bits(run_attn_dev(w, q_d, k_d, v_d, to_dev(w.block_tables), to_dev(lens),
                               max_context_len=128, check_tables=False))
    torch.cuda.synchronize()
    clamped = wl.custom([128, 90, 17, 0], 8, 2, seed=18, maxb=32)
    clamped.block_tables = w.block_tables
    check(clamped, q, k, v, got, "clamped to 128, negative length")
    assert not got.reshape(w.q_shape())[3].any()


def test_non_finite_values_in_valid_rows_stay_local(device):
    """NaN or Inf inside the rows a request does attend over propagates the way IEEE arithmetic
    has it and touches nothing else: a NaN in a K row makes the rows of that KV head's query
    group NaN in every dim, a NaN in one V element makes exactly that output dim NaN, an infinite
    V element leaves that dim non-finite; every other output element keeps its bits, and the NaN
    positions are the checker's."""
    lens = [300, 1000, 77, 2100]
    w = wl.custom(lens, 40, 8, seed=83, partition_size=256)
    q, k, v = wl.make_host_tensors(w)
    clean = run_attn(w, q, k, v).reshape(w.q_shape())
    G, B = 5, w.block_size
    NAN, INF = np.uint16(0x7FC0), np.uint16(0x7F80)
    k2, v2 = k.copy(), v.copy()
    where = lambda s, t: (w.block_tables[s, t // B], t % B)
    blk, slot = where(0, 5);    k2[blk, 1, slot, 40] = NAN        # request 0, KV head 1
    blk, slot = where(1, 700);  v2[blk, 0, slot, 17] = NAN        # request 1, KV head 0, dim 17
    blk, slot = where(3, 2099); v2[blk, 7, slot, 127] = INF       # request 3, KV head 7, dim 127
    blk, slot = where(3, 0);    k2[blk, 2, slot, 0] = NAN         # request 3, KV head 2
    got = run_attn(w, q, k2, v2).reshape(w.q_shape())
    gf = wl.bf16_bits_to_f64(got).reshape(w.q_shape())
    expect_nan = np.zeros(w.q_shape(), bool)
    expect_nan[0, 1 * G:2 * G, :] = True
    expect_nan[1, 0:G, 17] = True
    expect_nan[3, 2 * G:3 * G, :] = True
    inf_spot = np.zeros(w.q_shape(), bool)
    inf_spot[3, 7 * G:8 * G, 127] = True
    assert np.isnan(gf[expect_nan]).all()
    assert not np.isfinite(gf[inf_spot]).any()
    rest = ~(expect_nan | inf_spot)
    assert np.array_equal(got[rest], clean[rest])
    ref = oracle.paged_decode_attn(q, k2, v2, w.block_tables, w.context_lens, w.scale)
    assert np.array_equal(np.isnan(ref), expect_nan)
    assert np.isposinf(ref[inf_spot]).all()


@pytest.mark.parametrize("scale", [0.7, 8.0, -3.0])
def test_peaked_softmax(device, scale):
    """Scores hundreds of units apart (a softmax that is all but one-hot, and one turned upside down
    by a negative scale): the running maximum moves by far more than its lazy bound, old
    accumulators are rescaled by factors that underflow to zero, and the result still follows the
    checker."""
    w = wl.custom([300, 1000, 77, 2100, 1, 16], 40, 8, seed=85, partition_size=256)
    q, k, v = wl.make_host_tensors(w)
    got = to_bits(run_attn_dev(w, to_dev(q), to_dev(k), to_dev(v), to_dev(w.block_tables),
                               to_dev(w.context_lens), scale=scale))
    torch.cuda.synchronize()
    ref = oracle.paged_decode_attn(q, k, v, w.block_tables, w.context_lens, np.float32(scale))
    c = oracle.compare(got, ref)
    print(f"scale {scale}: {c}", flush=True)
    assert np.isfinite(wl.bf16_bits_to_f64(got)).all()
    assert c["rel_l2"] <= REL_L2 and c["worst_seq_rel_l2"] <= 2 * REL_L2, c
    from gpu_util import abs_error_within_bar
    assert abs_error_within_bar(got, ref), c       # near one-hot rows reproduce 4-sigma V elements


def test_stream_read_probe_runs_and_touches_nothing(device):
    """The measurement aid reads hashed slabs of two buffers and writes nothing: the buffers and a
    sentinel-filled sink are unchanged, whatever the block count (none, fewer than wavefronts, many)."""
    from paper_2602_11530_amd import binding as pkv
    g = torch.Generator(device=device)
    g.manual_seed(5)
    a = torch.randint(-2 ** 15, 2 ** 15, (3000 * 2048,), generator=g, device=device, dtype=torch.int16)
    b = torch.randint(-2 ** 15, 2 ** 15, (3000 * 2048,), generator=g, device=device, dtype=torch.int16)
    a0, b0 = a.clone(), b.clone()
    sink = torch.full((4,), 0x5A5A5A5A, dtype=torch.int32, device=device)
    for blocks in (0, 1, 77, 2048, 100_000):
        pkv.pkv_probe_stream_read(a, b, 3000, blocks, sink)      # 3000 slabs
    torch.cuda.synchronize()
    assert torch.equal(a, a0) and torch.equal(b, b0)
    assert (sink == 0x5A5A5A5A).all()
