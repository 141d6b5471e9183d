"""CPU-only pins for the fp64 checker: each test ties it to something that is
not itself — a dense brute force written here in numpy, a library attention
routine, closed forms and invariances — so that a dropped term, a wrong index or
a transposed operand in the checker fails at least one of them."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2602_11530_amd import workloads as wl


def depage(w, pool, s):
    """Dense [L, Hkv, D] float64 rows of request s (written independently of the
    checker: numpy fancy indexing, block-major)."""
    L = int(w.context_lens[s])
    nb = (L + w.block_size - 1) // w.block_size
    blocks = pool[w.block_tables[s, :nb]]                      # [nb, Hkv, B, D]
    rows = np.transpose(blocks, (0, 2, 1, 3)).reshape(nb * w.block_size, w.num_kv_heads,
                                                      w.head_dim)[:L]
    return wl.bf16_bits_to_f64(rows).reshape(L, w.num_kv_heads, w.head_dim)


def brute_force(w, q, k, v, scale):
    """softmax(scale * q K^T) V per request and head, dense numpy fp64."""
    out = np.zeros(w.q_shape(), dtype=np.float64)
    G = w.num_q_heads // w.num_kv_heads
    qf = wl.bf16_bits_to_f64(q).reshape(w.q_shape())
    for s in range(w.num_seqs):
        if w.context_lens[s] == 0:
            continue
        K = depage(w, k, s)
        V = depage(w, v, s)
        for h in range(w.num_q_heads):
            x = float(np.float32(scale)) * (K[:, h // G, :] @ qf[s, h])
            p = np.exp(x - x.max())
            p /= p.sum()
            out[s, h] = p @ V[:, h // G, :]
    return out


def run(w, q, k, v, scale=None):
    scale = w.scale if scale is None else scale
    return oracle.paged_decode_attn(q, k, v, w.block_tables, w.context_lens, scale)


def test_bf16_widening_matches_library():
    bits = np.arange(0, 65536, dtype=np.uint16)
    finite = ((bits >> 7) & 0xFF) != 0xFF
    bits = bits[finite]
    lib = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    assert np.array_equal(wl.bf16_bits_to_f64(bits), lib)
    # the checker's own widening: L = 1 returns V exactly (see below) on every pattern
    w = wl.custom([1], 1, 1, seed=3)
    for chunk in np.array_split(bits, len(bits) // 128 + 1):
        v = np.zeros(w.pool_shape(), np.uint16)
        v[w.block_tables[0, 0], 0, 0, :len(chunk)] = chunk
        q = np.zeros(w.q_shape(), np.uint16)
        got = run(w, q, v, v)
        assert np.array_equal(got[0, 0, :len(chunk)], wl.bf16_bits_to_f64(chunk))


def test_f32_to_bf16_matches_library_rounding():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 3,
                        np.array([1.00390625, 1.01171875, -1.00390625, 0.0, 65504.0],
                                 np.float32)])
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(wl.f32_to_bf16_bits(x), lib)


def test_brute_force_tiny_cfg1():
    w = wl.cfg1_tiny()
    assert w.num_seqs == 4 and w.num_q_heads == 8 and w.num_kv_heads == 2
    assert w.context_lens.min() >= 17 and w.context_lens.max() <= 300
    q, k, v = wl.make_host_tensors(w)
    ref = run(w, q, k, v)
    bf = brute_force(w, q, k, v, w.scale)
    assert np.abs(ref - bf).max() < 1e-12


@pytest.mark.parametrize("lens", [[1], [15, 16, 17], [31, 32, 33, 1, 0, 2], [511, 512, 513]])
def test_brute_force_edge_lengths(lens):
    w = wl.custom(lens, 10, 2, seed=11, num_pool_blocks=200)
    q, k, v = wl.make_host_tensors(w, poison_unused=True)
    ref = run(w, q, k, v)
    assert np.isfinite(ref).all()
    bf = brute_force(w, q, k, v, w.scale)
    assert np.abs(ref - bf).max() < 1e-12
    for s, L in enumerate(lens):
        if L == 0:
            assert not ref[s].any()


@pytest.mark.parametrize("D", [64, 256])
@pytest.mark.parametrize("B", [16, 32])
def test_brute_force_other_head_dims(D, B):
    """The checker is generic in the head dimension; head dims 64 and 256 against the same dense
    numpy brute force (and against torch's routine below), with the scale that goes with them."""
    w = wl.custom([33, 1, 0, 257, 16, 700], 12, 4, seed=17 + D, num_pool_blocks=90, head_dim=D,
                  block_size=B)
    assert w.scale == np.float32(1.0 / math.sqrt(D))
    q, k, v = wl.make_host_tensors(w, poison_unused=True)
    assert q.shape[-1] == D and k.shape[-1] == D
    ref = run(w, q, k, v)
    assert np.isfinite(ref).all() and not ref[2].any()
    assert np.abs(ref - brute_force(w, q, k, v, w.scale)).max() < 1e-12
    qf = torch.from_numpy(wl.bf16_bits_to_f64(q).reshape(w.q_shape()))
    for s in (0, 3, 5):
        K = torch.from_numpy(depage(w, k, s)).repeat_interleave(3, dim=1)
        V = torch.from_numpy(depage(w, v, s)).repeat_interleave(3, dim=1)
        o = torch.nn.functional.scaled_dot_product_attention(
            qf[s][:, None, :], K.permute(1, 0, 2), V.permute(1, 0, 2),
            scale=float(np.float32(w.scale)))
        assert np.abs(o[:, 0, :].numpy() - ref[s]).max() < 1e-12


def test_library_attention_medium():
    """torch's fp64 scaled_dot_product_attention on de-paged, head-repeated rows."""
    w = wl.custom([700, 45, 1300], 40, 8, seed=23)
    q, k, v = wl.make_host_tensors(w)
    ref = run(w, q, k, v)
    G = 5
    qf = torch.from_numpy(wl.bf16_bits_to_f64(q).reshape(w.q_shape()))
    for s in range(w.num_seqs):
        K = torch.from_numpy(depage(w, k, s)).repeat_interleave(G, dim=1)   # [L, Hq, D]
        V = torch.from_numpy(depage(w, v, s)).repeat_interleave(G, dim=1)
        o = torch.nn.functional.scaled_dot_product_attention(
            qf[s][:, None, :], K.permute(1, 0, 2), V.permute(1, 0, 2),
            scale=float(np.float32(w.scale)))
        assert np.abs(o[:, 0, :].numpy() - ref[s]).max() < 1e-12


def test_length_one_returns_v_exactly():
    w = wl.custom([1, 1, 1], 8, 2, seed=7, num_pool_blocks=50)
    q, k, v = wl.make_host_tensors(w, poison_unused=True)
    ref = run(w, q, k, v)
    for s in range(3):
        for h in range(8):
            want = wl.bf16_bits_to_f64(v[w.block_tables[s, 0], h // 4, 0])
            assert np.array_equal(ref[s, h], want)


def test_two_token_closed_form():
    """Scores ln 2 and 0 give weights 2/3 and 1/3; only head_dim element 0 of q
    and K is non-zero, so a transposed or mis-strided operand changes the result."""
    w = wl.custom([2], 2, 1, seed=1)
    D = w.head_dim
    pb = int(w.block_tables[0, 0])
    qf = np.zeros(w.q_shape(), np.float32)
    kf = np.zeros(w.pool_shape(), np.float32)
    vf = np.zeros(w.pool_shape(), np.float32)
    qf[0, 0, 0] = 1.0
    qf[0, 1, 3] = 2.0
    kf[pb, 0, 0, 0] = 1.0       # token 0, head 0 sees score scale*1
    kf[pb, 0, 1, 3] = 1.0       # token 1, head 1 sees score scale*2
    vf[pb, 0, 0, :] = 3.0
    vf[pb, 0, 1, :] = -6.0
    vf[pb, 0, 1, 5] = 12.0
    scale = np.float32(math.log(2.0))
    ref = oracle.paged_decode_attn(wl.f32_to_bf16_bits(qf), wl.f32_to_bf16_bits(kf),
                                   wl.f32_to_bf16_bits(vf), w.block_tables,
                                   w.context_lens, scale)
    a = math.exp(float(scale))            # head 0: weights a/(a+1), 1/(a+1)
    want0 = (a * 3.0 + 1.0 * -6.0) / (a + 1.0)
    b = math.exp(2.0 * float(scale))      # head 1: weights 1/(1+b), b/(1+b)
    want1 = (3.0 + b * -6.0) / (1.0 + b)
    assert abs(ref[0, 0, 1] - want0) < 1e-14 and abs(ref[0, 1, 1] - want1) < 1e-14
    assert abs(ref[0, 1, 5] - (3.0 + b * 12.0) / (1.0 + b)) < 1e-14
    assert abs(a - 2.0) < 1e-6            # fp32(ln 2): weights are 2/3, 1/3 to 1e-7
    assert abs(ref[0, 0, 0] - 0.0) < 1e-6


def test_scale_zero_is_mean_and_masks_hold():
    w = wl.custom([37, 16, 100], 8, 2, seed=9, num_pool_blocks=40)
    q, k, v = wl.make_host_tensors(w, poison_unused=True)
    ref = run(w, q, k, v, scale=0.0)
    for s in range(w.num_seqs):
        V = depage(w, v, s)
        for h in range(8):
            assert np.abs(ref[s, h] - V[:, h // 4, :].mean(0)).max() < 1e-13


def test_v_all_ones_gives_ones():
    """Weights sum to one: with V == 1 every output element is 1."""
    w = wl.cfg1_tiny()
    q, k, v = wl.make_host_tensors(w)
    v[:] = wl.f32_to_bf16_bits(np.ones(1, np.float32))[0]
    ref = run(w, q, k, v)
    assert np.abs(ref - 1.0).max() < 1e-14


def test_score_shift_invariance():
    """Adding one vector to every K row shifts all scores of a head alike."""
    w = wl.custom([90, 33], 4, 2, seed=13)
    rng = np.random.default_rng(2)
    # values on a 1/8 grid so that K + c is exact in bf16
    kf = rng.integers(-16, 17, size=w.pool_shape()).astype(np.float32) / 8
    cf = rng.integers(-8, 9, size=(w.head_dim,)).astype(np.float32) / 8
    qf = rng.integers(-8, 9, size=w.q_shape()).astype(np.float32) / 8
    _, _, v = wl.make_host_tensors(w)
    a = oracle.paged_decode_attn(wl.f32_to_bf16_bits(qf), wl.f32_to_bf16_bits(kf), v,
                                 w.block_tables, w.context_lens, w.scale)
    b = oracle.paged_decode_attn(wl.f32_to_bf16_bits(qf), wl.f32_to_bf16_bits(kf + cf), v,
                                 w.block_tables, w.context_lens, w.scale)
    assert np.abs(a - b).max() < 1e-12
    assert np.abs(a).max() > 1e-3


def test_split_context_merges_to_the_single_pass():
    """The split-K identity the GPU path relies on: cut a request's context at block boundaries
    into pieces, let the checker attend over each piece as a request of its own, and merge the
    normalised pieces with weights e^(m_p - M) Z_p (maximum and sum of each piece's scores from a
    dense numpy computation): the merged row equals the checker's single pass over the whole
    context.  A piece may also be empty (weight 0)."""
    lens = [300, 1000, 48]
    w = wl.custom(lens, 8, 2, seed=71)
    q, k, v = wl.make_host_tensors(w)
    whole = run(w, q, k, v)
    G, B = w.num_q_heads // w.num_kv_heads, w.block_size
    qf = wl.bf16_bits_to_f64(q).reshape(w.q_shape())
    for cuts in ([128], [16, 32, 512], [48], [0]):
        for s, L in enumerate(lens):
            edges = [0] + [c for c in cuts if c < L] + [L]
            K = depage(w, k, s)
            num = np.zeros((w.num_q_heads, w.head_dim))
            den = np.zeros(w.num_q_heads)
            stats = []
            for a0, a1 in zip(edges[:-1], edges[1:]):
                # the piece [a0, a1) as a request: its table row starts at block a0 / B
                t = np.full((1, w.max_blocks_per_seq), -1, np.int32)
                nb = (a1 - a0 + B - 1) // B
                t[0, :nb] = w.block_tables[s, a0 // B:a0 // B + nb]
                piece = oracle.paged_decode_attn(q[s:s + 1], k, v, t, np.array([a1 - a0], np.int32), w.scale)[0]
                x = float(np.float32(w.scale)) * np.einsum("tkd,kgd->kgt", K[a0:a1],
                                                           qf[s].reshape(w.num_kv_heads, G, -1))
                x = x.reshape(w.num_q_heads, a1 - a0)
                m = x.max(axis=1) if a1 > a0 else np.full(w.num_q_heads, -np.inf)
                Z = np.exp(x - m[:, None]).sum(axis=1) if a1 > a0 else np.zeros(w.num_q_heads)
                stats.append((m, Z, piece))
            M = np.max([m for m, _, _ in stats], axis=0)
            for m, Z, piece in stats:
                wgt = np.where(np.isneginf(m), 0.0, np.exp(m - M)) * Z
                num += wgt[:, None] * piece
                den += wgt
            assert np.abs(num / den[:, None] - whole[s]).max() < 1e-12, (cuts, s)


def test_paging_invariance():
    """Permute the physical blocks and rewrite the tables: identical result."""
    w = wl.cfg1_tiny()
    q, k, v = wl.make_host_tensors(w)
    ref = run(w, q, k, v)
    rng = np.random.default_rng(99)
    perm = rng.permutation(w.num_pool_blocks)       # new id of old block i = perm[i]
    k2, v2 = np.empty_like(k), np.empty_like(v)
    k2[perm], v2[perm] = k, v
    t2 = np.where(w.block_tables >= 0, perm[np.clip(w.block_tables, 0, None)], -1).astype(np.int32)
    ref2 = oracle.paged_decode_attn(q, k2, v2, t2, w.context_lens, w.scale)
    assert np.array_equal(ref, ref2)


def test_gqa_equals_mha_with_repeated_kv():
    w = wl.cfg1_tiny()
    q, k, v = wl.make_host_tensors(w)
    ref = run(w, q, k, v)
    G = w.num_q_heads // w.num_kv_heads
    k_rep = np.repeat(k, G, axis=1)
    v_rep = np.repeat(v, G, axis=1)
    ref_mha = oracle.paged_decode_attn(q, k_rep, v_rep, w.block_tables, w.context_lens, w.scale)
    assert np.array_equal(ref, ref_mha)


def test_batch_independence():
    w = wl.cfg1_tiny()
    q, k, v = wl.make_host_tensors(w)
    ref = run(w, q, k, v)
    idx = [2, 0]
    sub = wl.subset(w, idx)
    ref_sub = oracle.paged_decode_attn(q[idx], k, v, sub.block_tables, sub.context_lens, w.scale)
    assert np.array_equal(ref_sub, ref[idx])


def test_unused_table_entries_never_read():
    w = wl.cfg1_tiny()
    q, k, v = wl.make_host_tensors(w)
    ref = run(w, q, k, v)
    t = w.block_tables.copy()
    t[t < 0] = w.num_pool_blocks + 12345
    ref2 = oracle.paged_decode_attn(q, k, v, t, w.context_lens, w.scale)
    assert np.array_equal(ref, ref2)
    t[0, 0] = w.num_pool_blocks      # a *used* entry out of range is rejected
    with pytest.raises(ValueError):
        oracle.paged_decode_attn(q, k, v, t, w.context_lens, w.scale)


def test_gather_scatter_against_fancy_indexing():
    rng = np.random.default_rng(4)
    pool = rng.integers(0, 65536, size=(50, 2, 16, 128)).astype(np.uint16)
    ids = rng.permutation(50)[:17].astype(np.int32)
    st = oracle.kv_blocks_gather(pool, ids)
    assert np.array_equal(st, pool[ids])
    new_ids = rng.permutation(50)[:17].astype(np.int32)
    out = oracle.kv_blocks_scatter(st, pool, new_ids)
    want = pool.copy()
    want[new_ids] = st
    assert np.array_equal(out, want)
    untouched = np.setdiff1d(np.arange(50), new_ids)
    assert np.array_equal(out[untouched], pool[untouched])
    assert oracle.kv_blocks_gather(pool, np.zeros(0, np.int32)).shape[0] == 0
    with pytest.raises(ValueError):
        oracle.kv_blocks_scatter(st, pool, np.array([1] * 17, np.int32))
    with pytest.raises(ValueError):
        oracle.kv_blocks_gather(pool, np.array([50], np.int32))


def test_move_against_fancy_indexing():
    rng = np.random.default_rng(14)
    src = rng.integers(0, 65536, size=(40, 2, 16, 128)).astype(np.uint16)
    dst = rng.integers(0, 65536, size=(25, 2, 16, 128)).astype(np.uint16)
    a = rng.permutation(40)[:11].astype(np.int32)
    b = rng.permutation(25)[:11].astype(np.int32)
    out = oracle.kv_blocks_move(src, a, dst, b)
    want = dst.copy()
    want[b] = src[a]
    assert np.array_equal(out, want) and (out != dst).any()
    # the same as a gather followed by a scatter
    assert np.array_equal(out, oracle.kv_blocks_scatter(oracle.kv_blocks_gather(src, a), dst, b))
    assert np.array_equal(oracle.kv_blocks_move(src, a[:0], dst, b[:0]), dst)
    with pytest.raises(ValueError):
        oracle.kv_blocks_move(src, a, dst, np.array([3] * 11, np.int32))     # a destination twice
    with pytest.raises(ValueError):
        oracle.kv_blocks_move(src, np.array([40], np.int32), dst, b[:1])     # source out of range


def test_migration_round_trip_keeps_attention():
    w = wl.cfg1_tiny()
    q, k, v = wl.make_host_tensors(w)
    ref = run(w, q, k, v)
    mig = wl.make_migration(w, 0.25)
    k2 = oracle.kv_blocks_scatter(oracle.kv_blocks_gather(k, mig.old_ids), k, mig.new_ids)
    v2 = oracle.kv_blocks_scatter(oracle.kv_blocks_gather(v, mig.old_ids), v, mig.new_ids)
    ref2 = oracle.paged_decode_attn(q, k2, v2, mig.tables_after, w.context_lens, w.scale)
    assert np.array_equal(ref, ref2)


def test_kv_append_against_indexing():
    w = wl.custom([1, 16, 17, 0, 300, 33], 8, 2, seed=31, num_pool_blocks=60)
    rng = np.random.default_rng(6)
    _, k, v = wl.make_host_tensors(w)
    k_new = rng.integers(0, 65536, size=(w.num_seqs, 2, 128)).astype(np.uint16)
    v_new = rng.integers(0, 65536, size=(w.num_seqs, 2, 128)).astype(np.uint16)
    k2, v2 = oracle.kv_append(k_new, v_new, k, v, w.block_tables, w.context_lens)
    wk, wv = k.copy(), v.copy()
    for s, L in enumerate(w.context_lens):
        if L > 0:
            pb = w.block_tables[s, (L - 1) // 16]
            wk[pb, :, (L - 1) % 16, :] = k_new[s]
            wv[pb, :, (L - 1) % 16, :] = v_new[s]
    assert np.array_equal(k2, wk) and np.array_equal(v2, wv)
    assert (k2 != k).any() and np.array_equal(k, wl.make_host_tensors(w)[1])   # input not modified
    # the appended row is the one attention sees last: with a huge score on it the output is its V row
    q = np.zeros(w.q_shape(), np.uint16)
    q[:] = wl.f32_to_bf16_bits(np.full(1, 8.0, np.float32))[0]
    k_hot = np.full_like(k_new, wl.f32_to_bf16_bits(np.full(1, 8.0, np.float32))[0])
    v_new = wl.normal_bf16(rng, v_new.shape)
    k3, v3 = oracle.kv_append(k_hot, v_new, np.zeros_like(k), v, w.block_tables, w.context_lens)
    ref = oracle.paged_decode_attn(q, k3, v3, w.block_tables, w.context_lens, 1.0)
    for s, L in enumerate(w.context_lens):
        if L > 0:
            assert np.abs(ref[s, 0] - wl.bf16_bits_to_f64(v_new[s, 0])).max() < 1e-6


# ---- the comparison every tolerance assertion goes through ------------------------------

def _bits(values):
    """bf16 bit patterns of values that bf16 holds exactly (checked), via torch."""
    t = torch.tensor(values, dtype=torch.float64)
    b = t.to(torch.bfloat16)
    assert torch.equal(b.to(torch.float64), t), "test values must be exact in bf16"
    return b.view(torch.int16).numpy().view(np.uint16)


def test_compare_known_errors():
    """Hand-made arrays with errors known in advance."""
    ref = np.array([[[1.0, 2.0], [3.0, 4.0]],
                    [[0.5, -0.5], [8.0, -16.0]]])            # [S=2, Hq=2, D=2]
    exact = oracle.compare(_bits(ref.tolist()), ref)
    assert exact == {"max_abs": 0.0, "rel_l2": 0.0, "worst_seq_rel_l2": 0.0}
    # one element of request 0 off by 0.5, one of request 1 off by 0.25
    got = [[[1.0, 2.5], [3.0, 4.0]], [[0.5, -0.25], [8.0, -16.0]]]
    c = oracle.compare(_bits(got), ref)
    assert c["max_abs"] == 0.5
    # ||diff|| = sqrt(0.25 + 0.0625); ||ref||^2 = 1 + 4 + 9 + 16 + 0.25 + 0.25 + 64 + 256
    assert c["rel_l2"] == pytest.approx(math.sqrt(0.3125) / math.sqrt(350.5), rel=1e-14)
    # per request: 0.5 / sqrt(30) against 0.25 / sqrt(320.5): request 0 is the worst
    assert c["worst_seq_rel_l2"] == pytest.approx(0.5 / math.sqrt(30.0), rel=1e-14)
    # the same errors the other way round: now request 1 is the worst, and its own norm is used
    got = [[[1.0, 2.0], [3.0, 4.0]], [[2.5, -0.5], [8.0, -16.0]]]
    c = oracle.compare(_bits(got), ref)
    assert c["max_abs"] == 2.0
    assert c["worst_seq_rel_l2"] == pytest.approx(2.0 / math.sqrt(320.5), rel=1e-14)
    assert c["rel_l2"] == pytest.approx(2.0 / math.sqrt(350.5), rel=1e-14)
    # a flat array of bits is read in the reference's row-major order
    flat = _bits(got).reshape(-1)
    assert oracle.compare(flat, ref) == c
    # sign matters: -x against x is an error of 2|x|
    c = oracle.compare(_bits((-ref).tolist()), ref)
    assert c["max_abs"] == 32.0 and c["rel_l2"] == pytest.approx(2.0, rel=1e-14)


def test_compare_reads_bf16_bit_patterns():
    ref = np.array([[[1.0, -2.0, 0.0, 0.099609375]]])
    bits = np.array([[[0x3F80, 0xC000, 0x8000, 0x3DCC]]], dtype=np.uint16)   # 1, -2, -0, 0.099609375
    assert oracle.compare(bits, ref)["max_abs"] == 0.0
    bits[0, 0, 3] = 0x3DCD                                    # one unit in the last place up: 2^-11
    assert oracle.compare(bits, ref)["max_abs"] == 2.0 ** -11


def test_compare_zero_reference_and_empty_batch():
    """A reference that is zero everywhere (requests of length 0) has no relative scale: the
    measure falls back to the absolute norm of the difference, and rows whose reference is
    zero take no part in the per-request maximum."""
    ref = np.zeros((2, 1, 2))
    assert oracle.compare(_bits([[[0.0, 0.0]], [[0.0, 0.0]]]), ref) == \
        {"max_abs": 0.0, "rel_l2": 0.0, "worst_seq_rel_l2": 0.0}
    c = oracle.compare(_bits([[[0.0, 3.0]], [[4.0, 0.0]]]), ref)
    assert c["max_abs"] == 4.0 and c["rel_l2"] == 5.0 and c["worst_seq_rel_l2"] == 0.0
    ref = np.array([[[0.0, 0.0]], [[1.0, 1.0]]])
    c = oracle.compare(_bits([[[0.0, 0.0]], [[1.0, 1.5]]]), ref)
    assert c["worst_seq_rel_l2"] == pytest.approx(0.5 / math.sqrt(2.0), rel=1e-14)
    assert oracle.compare(np.zeros((0, 4, 8), np.uint16), np.zeros((0, 4, 8))) == \
        {"max_abs": 0.0, "rel_l2": 0.0, "worst_seq_rel_l2": 0.0}


def test_compare_rejects_wrong_outputs_at_the_bar():
    """Outputs that are wrong in the ways a kernel can be wrong land above the parity bar
    (max-abs 1e-2, relative L2 5e-3), and a correctly rounded output lands below it."""
    w = wl.custom([40, 300, 77], 8, 2, seed=31, num_pool_blocks=64)
    q, k, v = wl.make_host_tensors(w)
    ref = oracle.paged_decode_attn(q, k, v, w.block_tables, w.context_lens, w.scale)
    rounded = torch.from_numpy(ref).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    good = oracle.compare(rounded, ref)
    assert good["max_abs"] <= 1e-2 and 5e-4 < good["rel_l2"] <= 5e-3 and good["worst_seq_rel_l2"] <= 5e-3
    wrong = {
        "heads swapped": rounded[:, ::-1, :],
        "requests rotated": np.roll(rounded, 1, axis=0),
        "dims reversed": rounded[:, :, ::-1],
        "truncated instead of rounded, then one ulp low": rounded - np.uint16(1),
        "one request zero": np.concatenate([rounded[:1] * np.uint16(0), rounded[1:]]),
    }
    for what, bits in wrong.items():
        c = oracle.compare(np.ascontiguousarray(bits), ref)
        assert c["rel_l2"] > 5e-3 or c["max_abs"] > 1e-2, what
    # an error confined to the shortest request still shows in the per-request figure
    bits = rounded.copy()
    bits[0, 0, :4] ^= np.uint16(0x0040)                       # flips a mantissa bit: ~25-50 % off
    c = oracle.compare(bits, ref)
    assert c["worst_seq_rel_l2"] > 5e-3 and c["worst_seq_rel_l2"] > c["rel_l2"]


# ---- 8-bit (E4M3) KV pools --------------------------------------------------------------

def e4m3_values(bits: np.ndarray) -> np.ndarray:
    """The library's decode of E4M3 bytes (torch's float8_e4m3fn), as float64."""
    return torch.from_numpy(np.ascontiguousarray(bits)).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def test_e4m3_decode_every_byte():
    got = np.array([oracle.e4m3(b) for b in range(256)])
    want = e4m3_values(np.arange(256, dtype=np.uint8))
    nan = np.isnan(want)
    assert sorted(np.nonzero(nan)[0].tolist()) == [0x7F, 0xFF]
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))
    # the format's landmarks, written out: 1, the largest finite value, the smallest subnormal,
    # the smallest normal, and the seven subnormals m * 2^-9
    assert oracle.e4m3(0x38) == 1.0 and oracle.e4m3(0x7E) == 448.0 and oracle.e4m3(0xFE) == -448.0
    assert oracle.e4m3(0x01) == 2.0 ** -9 and oracle.e4m3(0x08) == 2.0 ** -6
    assert [oracle.e4m3(m) for m in range(8)] == [m * 2.0 ** -9 for m in range(8)]
    assert oracle.e4m3(0x3C) == 1.5 and oracle.e4m3(0x40) == 2.0 and oracle.e4m3(0xC0) == -2.0


def brute_force_values(w, qf, Kf, Vf, scale):
    """Dense softmax(scale * q K^T) V on pools given as float64 values."""
    out = np.zeros(w.q_shape(), dtype=np.float64)
    G = w.num_q_heads // w.num_kv_heads

    def rows(pool, s):
        L = int(w.context_lens[s])
        nb = (L + w.block_size - 1) // w.block_size
        blocks = pool[w.block_tables[s, :nb]]
        return np.transpose(blocks, (0, 2, 1, 3)).reshape(nb * w.block_size, w.num_kv_heads, w.head_dim)[:L]

    for s in range(w.num_seqs):
        if w.context_lens[s] == 0:
            continue
        K, V = rows(Kf, s), rows(Vf, s)
        for h in range(w.num_q_heads):
            x = float(np.float32(scale)) * (K[:, h // G, :] @ qf[s, h])
            p = np.exp(x - x.max())
            out[s, h] = (p / p.sum()) @ V[:, h // G, :]
    return out


@pytest.mark.parametrize("B", [16, 64])
def test_fp8kv_attention_against_brute_force(B):
    ks, vs = np.float32(0.013), np.float32(0.021)
    w = wl.custom([33, 1, 0, 257, 16, 700, 15], 10, 2, seed=61, num_pool_blocks=90, block_size=B)
    q, k8, v8 = wl.make_host_tensors_fp8(w, ks, vs, poison_unused=True)
    assert k8.dtype == np.uint8 and (k8 == 0x7F).any() and (v8 == 0xFF).any()
    ref = oracle.paged_decode_attn_fp8kv(q, k8, v8, w.block_tables, w.context_lens, w.scale, ks, vs)
    assert np.isfinite(ref).all() and not ref[2].any()
    qf = wl.bf16_bits_to_f64(q).reshape(w.q_shape())
    Kf = np.nan_to_num(e4m3_values(k8)) * float(ks)       # the poison never enters a valid row
    Vf = np.nan_to_num(e4m3_values(v8)) * float(vs)
    bf = brute_force_values(w, qf, Kf, Vf, w.scale)
    assert np.abs(ref - bf).max() < 1e-12
    # the values really are a unit-variance pool seen through the scales
    assert 0.9 < Kf[w.block_tables[5, 0], :, :, :].std() < 1.1


def test_fp8kv_equals_bf16_function_on_the_same_values():
    """Every E4M3 value is a bf16 value: with unit scales the 8-bit function and the bf16
    function must agree on a pool holding the same numbers; and the scales act as factors on
    the scores and on the output."""
    w = wl.custom([300, 45, 1, 64], 12, 4, seed=62, num_pool_blocks=40)
    q, k8, v8 = wl.make_host_tensors_fp8(w, 0.02, 0.02)
    as_bf16 = lambda b: torch.from_numpy(e4m3_values(b)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    kb, vb = as_bf16(k8), as_bf16(v8)
    assert np.array_equal(wl.bf16_bits_to_f64(kb), e4m3_values(k8))     # the widening is exact
    a = oracle.paged_decode_attn_fp8kv(q, k8, v8, w.block_tables, w.context_lens, 0.01, 1.0, 1.0)
    b = oracle.paged_decode_attn(q, kb, vb, w.block_tables, w.context_lens, 0.01)
    assert np.abs(a - b).max() < 1e-13 * np.abs(b).max()
    # k_scale multiplies the scores: (scale, 4 k) == (4 scale, k); v_scale multiplies the rows
    c = oracle.paged_decode_attn_fp8kv(q, k8, v8, w.block_tables, w.context_lens, 0.0025, 4.0, 1.0)
    assert np.abs(a - c).max() < 1e-13 * np.abs(a).max()
    d = oracle.paged_decode_attn_fp8kv(q, k8, v8, w.block_tables, w.context_lens, 0.01, 1.0, 3.0)
    assert np.abs(d - 3.0 * a).max() < 1e-13 * np.abs(a).max()
    # one token: the row is v_scale times the decoded bytes
    one = oracle.paged_decode_attn_fp8kv(q, k8, v8, w.block_tables, w.context_lens, 0.01, 1.0, 0.5)
    assert np.array_equal(one[2, 5], 0.5 * e4m3_values(v8[w.block_tables[2, 0], 5 // 3, 0]))


def test_to_e4m3_against_library_rounding():
    """fp32 -> E4M3 on every finite bf16 value (as fp32) and on a dense set of fp32 values around
    every rounding boundary: equal to torch's conversion wherever that is finite, and saturated
    to +-448 where torch overflows to NaN."""
    bits = np.arange(65536, dtype=np.uint32)
    vals = (bits << np.uint32(16)).view(np.float32)
    vals = vals[np.isfinite(vals)]
    # midpoints between neighbouring E4M3 values, and their fp32 neighbours on either side
    grid = np.array(sorted({oracle.e4m3(b) for b in range(0x7F)}), dtype=np.float64)
    mids = ((grid[1:] + grid[:-1]) / 2).astype(np.float32)
    around = np.concatenate([mids, np.nextafter(mids, np.float32(np.inf)), np.nextafter(mids, np.float32(-np.inf))])
    vals = np.concatenate([vals, around, -around, np.float32([448, 449, 463.9, 464, 465, 1e9, -1e9, 3e38])])
    lib = torch.from_numpy(vals).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.to_e4m3(v) for v in vals], dtype=np.uint8)
    overflow = (lib & 0x7F) == 0x7F
    assert np.array_equal(got[~overflow], lib[~overflow])
    assert (np.abs(vals[overflow]) > 448).all()
    assert np.array_equal(got[overflow], np.where(vals[overflow] > 0, 0x7E, 0xFE).astype(np.uint8))
    # ties go to the even mantissa: 1.0625 is halfway between 1 (0x38) and 1.125 (0x39)
    assert oracle.to_e4m3(1.0625) == 0x38 and oracle.to_e4m3(1.1875) == 0x3A
    assert oracle.to_e4m3(2.0 ** -10) == 0x00 and oracle.to_e4m3(3 * 2.0 ** -10) == 0x02   # subnormal ties
    assert oracle.to_e4m3(-0.0) == 0x80 and oracle.to_e4m3(float("nan")) & 0x7F == 0x7F
    # decode(encode(x)) is the nearest grid point
    for v in np.float32([0.3, -1.7, 5.5, 100.0, 0.004, 447.0]):
        d = oracle.e4m3(oracle.to_e4m3(v))
        assert abs(d - v) == np.abs(grid - abs(v)).min()


def test_kv_append_fp8_against_indexing():
    w = wl.custom([1, 16, 17, 0, 300, 33], 12, 4, seed=41, num_pool_blocks=60)
    rng = np.random.default_rng(8)
    ks, vs = np.float32(0.0134), np.float32(0.02)
    _, k8, v8 = wl.make_host_tensors_fp8(w, ks, vs)
    k_new, v_new = wl.normal_bf16(rng, (w.num_seqs, 4, 128)), wl.normal_bf16(rng, (w.num_seqs, 4, 128))
    k_new[0, 0, :4] = wl.f32_to_bf16_bits(np.float32([100.0, -100.0, 0.0, 6.0]))   # saturates at 448 * scale
    ka, va = oracle.kv_append_fp8(k_new, v_new, k8, v8, w.block_tables, w.context_lens, ks, vs)
    q = lambda x, s: torch.from_numpy(np.clip(wl.bf16_bits_to_f64(x).astype(np.float32) / s, -448, 448)) \
        .to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    wk, wv = k8.copy(), v8.copy()
    for s, L in enumerate(w.context_lens):
        if L > 0:
            wk[w.block_tables[s, (L - 1) // 16], :, (L - 1) % 16] = q(k_new[s], ks)
            wv[w.block_tables[s, (L - 1) // 16], :, (L - 1) % 16] = q(v_new[s], vs)
    assert np.array_equal(ka, wk) and np.array_equal(va, wv)
    assert ka[w.block_tables[0, 0], 0, 0, 0] == 0x7E and ka[w.block_tables[0, 0], 0, 0, 1] == 0xFE
