"""GPU parity of kv_append (bit-exact) and of a short decode loop: append the new
token's K,V rows, then attend — the order every decode step runs in (paper
Section II-A)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_11530_amd import binding as pkv
from paper_2602_11530_amd import workloads as wl

from gpu_util import MAX_ABS, REL_L2, assert_launchable, run_attn_dev, shape_of, to_bits, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.expects_id_faults
def test_append_bit_exact_and_skips(device, id_faults):
    w = wl.custom([1, 16, 17, 0, 300, 33, 512, 513], 40, 8, seed=41, num_pool_blocks=120)
    assert_launchable(w)
    rng = np.random.default_rng(8)
    _, k, v = wl.make_host_tensors(w)
    k_new = rng.integers(0, 65536, size=(w.num_seqs, 8, 128)).astype(np.uint16)
    v_new = rng.integers(0, 65536, size=(w.num_seqs, 8, 128)).astype(np.uint16)
    k_d, v_d = to_dev(k), to_dev(v)
    pkv.kv_append(to_dev(k_new), to_dev(v_new), k_d, v_d, to_dev(w.block_tables),
                  to_dev(w.context_lens), shape_of(w))
    torch.cuda.synchronize()
    wk, wv = oracle.kv_append(k_new, v_new, k, v, w.block_tables, w.context_lens)
    assert np.array_equal(to_bits(k_d).reshape(k.shape), wk)
    assert np.array_equal(to_bits(v_d).reshape(v.shape), wv)
    assert int(id_faults.item()) == 0
    # a table entry outside the pool is skipped (and reported), everything else still written
    bad = w.block_tables.copy()
    bad[4, (300 - 1) // 16] = w.num_pool_blocks + 5
    bad[1, 0] = -3
    k_d, v_d = to_dev(k), to_dev(v)
    pkv.kv_append(to_dev(k_new), to_dev(v_new), k_d, v_d, to_dev(bad), to_dev(w.context_lens),
                  shape_of(w))
    torch.cuda.synchronize()
    assert int(id_faults.item()) == 2      # one report per skipped request
    lens_ok = w.context_lens.copy()
    lens_ok[[4, 1]] = 0
    wk, wv = oracle.kv_append(k_new, v_new, k, v, w.block_tables, lens_ok)
    assert np.array_equal(to_bits(k_d).reshape(k.shape), wk)
    assert np.array_equal(to_bits(v_d).reshape(v.shape), wv)


def test_decode_loop_append_then_attend(device):
    """Three decode steps of a mixed batch: lengths grow by one, the new rows are
    appended through the library, attention is checked against the oracle run on
    pools the oracle appended to itself."""
    final = np.array([20, 48, 515, 1300, 3], np.int32)
    w = wl.custom(final, 40, 8, seed=43, num_pool_blocks=200)   # tables cover the final lengths
    rng = np.random.default_rng(12)
    q, k, v = wl.make_host_tensors(w)
    k_d, v_d, t_d = to_dev(k), to_dev(v), to_dev(w.block_tables)
    k_h, v_h = k.copy(), v.copy()
    for step, back in enumerate((2, 1, 0)):
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
        ref = oracle.paged_decode_attn(q, k_h, v_h, w.block_tables, w.context_lens, w.scale)
        c = oracle.compare(to_bits(out), ref)
        print(f"decode step {step}: {c}", flush=True)
        assert c["max_abs"] <= MAX_ABS and c["rel_l2"] <= REL_L2, c


def test_append_honours_the_length_bound(device):
    """With max_context_len below a request's length the new row lands at the bound's last
    position, where attention with the same bound will look for it."""
    w = wl.custom([300, 90], 8, 2, seed=19, maxb=32)
    rng = np.random.default_rng(19)
    _, k, v = wl.make_host_tensors(w)
    k_new, v_new = wl.normal_bf16(rng, (2, 2, 128)), wl.normal_bf16(rng, (2, 2, 128))
    k_d, v_d = to_dev(k), to_dev(v)
    pkv.kv_append(to_dev(k_new), to_dev(v_new), k_d, v_d, to_dev(w.block_tables),
                  to_dev(w.context_lens), shape_of(w, max_context_len=128))
    torch.cuda.synchronize()
    wk, wv = oracle.kv_append(k_new, v_new, k, v, w.block_tables, np.array([128, 90], np.int32))
    assert np.array_equal(to_bits(k_d).reshape(k.shape), wk)
    assert np.array_equal(to_bits(v_d).reshape(v.shape), wv)
