"""The entry point that allocates nothing (`paged_decode_attn_static`): same rows,
bit for bit, as `paged_decode_attn` with a caller-owned workspace, on two calls in
a row that share the library's fixed workspace, the second with a smaller batch."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_11530_amd import binding as pkv
from paper_2602_11530_amd import workloads as wl

from gpu_util import MAX_ABS, REL_L2, assert_launchable, run_attn_dev, shape_of, to_bits, to_dev

pytestmark = pytest.mark.gpu


def static_call(w, dev, P):
    q_d, k_d, v_d, t_d, l_d = dev
    out = torch.full(w.q_shape(), 0x7FC1, dtype=torch.int16, device=q_d.device)
    shape = shape_of(w, P, int(w.context_lens.max()))
    pkv.paged_decode_attn_static(q_d, k_d, v_d, t_d, l_d, float(w.scale), out, shape)
    return out


@pytest.mark.parametrize("P", [0, 512])
def test_static_workspace_call_matches_the_caller_workspace_call(device, P):
    big = wl.custom([4100, 17, 2049, 1, 999, 6000, 1024, 96, 513, 3000], 40, 8, seed=77,
                    num_pool_blocks=1400)
    small = wl.custom([300, 33, 1], 40, 8, seed=78, num_pool_blocks=64)
    results = []
    for w in (big, small):            # the second call is smaller and reuses the same array
        assert_launchable(w)
        rng = np.random.default_rng(w.seed)
        host = (wl.normal_bf16(rng, w.q_shape()), wl.normal_bf16(rng, w.pool_shape()),
                wl.normal_bf16(rng, w.pool_shape()))
        dev = tuple(to_dev(x) for x in host + (w.block_tables, w.context_lens))
        shape = shape_of(w, P, int(w.context_lens.max()))
        assert pkv.pkv_attn_workspace_bytes(shape) <= pkv.STATIC_WORKSPACE_BYTES
        print(f"static call: {w.num_seqs} requests, P={P}", flush=True)
        got = static_call(w, dev, P)
        want = run_attn_dev(w, *dev, partition_size=P, max_context_len=int(w.context_lens.max()))
        torch.cuda.synchronize()
        assert torch.equal(got, want), "static-workspace call differs from the workspace call"
        ref = oracle.paged_decode_attn(*host, w.block_tables, w.context_lens, w.scale)
        c = oracle.compare(to_bits(got), ref)
        assert c["max_abs"] <= MAX_ABS and c["rel_l2"] <= REL_L2, c
        results.append(got)
    # the big batch again, after the small one left its records in the array
    w = big
    rng = np.random.default_rng(w.seed)
    host = (wl.normal_bf16(rng, w.q_shape()), wl.normal_bf16(rng, w.pool_shape()),
            wl.normal_bf16(rng, w.pool_shape()))
    dev = tuple(to_dev(x) for x in host + (w.block_tables, w.context_lens))
    again = static_call(w, dev, P)
    torch.cuda.synchronize()
    assert torch.equal(again, results[0])


def test_static_workspace_limit_is_enforced(device):
    """A shape whose workspace exceeds the fixed array is refused before any launch."""
    shape = pkv.make_shape(2048, 128, 8, 4, 64)     # 2048 requests x 8 KV heads of 16-head records
    assert pkv.pkv_attn_workspace_bytes(shape) > pkv.STATIC_WORKSPACE_BYTES
    t = torch.zeros(16, dtype=torch.int16, device=device)
    with pytest.raises(pkv.PkvError) as e:
        pkv.paged_decode_attn_static(t, t, t, t, t, 1.0, t, shape)
    assert e.value.status == pkv.PKV_ERR_WORKSPACE


def test_static_workspace_call_under_graph_capture(device):
    """The callers this entry point is for: a decode step (append + attention) recorded into a HIP
    graph with no workspace to carry around, replayed for four steps with growing lengths and fresh
    inputs; every replay equals the same step run eagerly with a caller-owned workspace and is
    within tolerance of the oracle.  The entry point is called once before the capture, as the
    header asks (its first call on a device looks up the array's address)."""
    n_steps = 4
    final = np.array([40, 16 * 9 + 1, 1030, 5, 2300, 64], np.int32)
    w = wl.custom(final, 40, 8, seed=58, num_pool_blocks=330)
    rng = np.random.default_rng(58)
    _, k_h, v_h = wl.make_host_tensors(w)
    k_g, v_g = to_dev(k_h), to_dev(v_h)
    k_e, v_e = k_g.clone(), v_g.clone()
    t_d = to_dev(w.block_tables)
    shape = shape_of(w)
    assert pkv.pkv_attn_workspace_bytes(shape) <= pkv.STATIC_WORKSPACE_BYTES
    ws = torch.empty(pkv.pkv_attn_workspace_bytes(shape), dtype=torch.uint8, device=device)
    S, Hkv = w.num_seqs, w.num_kv_heads
    lens_d = to_dev(final - n_steps)
    q_s = torch.zeros(w.q_shape(), dtype=torch.int16, device=device)
    kn_s = torch.zeros((S, Hkv, 128), dtype=torch.int16, device=device)
    vn_s = torch.zeros((S, Hkv, 128), dtype=torch.int16, device=device)
    out_s = torch.full(w.q_shape(), 0x7FC1, dtype=torch.int16, device=device)
    # first call outside the capture
    pkv.paged_decode_attn_static(q_s, k_g, v_g, t_d, lens_d, float(w.scale), out_s, shape)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pkv.kv_append(kn_s, vn_s, k_g, v_g, t_d, lens_d, shape)
        pkv.paged_decode_attn_static(q_s, k_g, v_g, t_d, lens_d, float(w.scale), out_s, shape)
    torch.cuda.synchronize()
    assert torch.equal(k_g, k_e), "capture must execute nothing"

    for step in range(n_steps):
        lens_d.add_(1)
        w.context_lens = final - n_steps + step + 1
        assert_launchable(w)
        q, kn, vn = wl.normal_bf16(rng, w.q_shape()), wl.normal_bf16(rng, (S, Hkv, 128)), \
            wl.normal_bf16(rng, (S, Hkv, 128))
        q_s.copy_(to_dev(q)); kn_s.copy_(to_dev(kn)); vn_s.copy_(to_dev(vn))
        out_s.fill_(0x7FC1)
        graph.replay()
        torch.cuda.synchronize()
        replayed = out_s.clone()
        eager = torch.full(w.q_shape(), 0x7FC1, dtype=torch.int16, device=device)
        pkv.kv_append(kn_s, vn_s, k_e, v_e, t_d, lens_d, shape)
        pkv.paged_decode_attn(q_s, k_e, v_e, t_d, lens_d, float(w.scale), eager, shape, ws)
        torch.cuda.synchronize()
        assert torch.equal(replayed, eager), f"step {step}: replay != eager"
        assert torch.equal(k_g, k_e) and torch.equal(v_g, v_e)
        k_h, v_h = oracle.kv_append(kn, vn, k_h, v_h, w.block_tables, w.context_lens)
        ref = oracle.paged_decode_attn(q, k_h, v_h, w.block_tables, w.context_lens, w.scale)
        c = oracle.compare(to_bits(replayed), ref)
        assert c["max_abs"] <= MAX_ABS and c["rel_l2"] <= REL_L2, (step, c)
