"""The multi-layer attention call, and a decode step captured in a HIP graph.

A request has the same length and block ids in every layer, so one table serves
all layers of a decode iteration (paper Section II-A); the launches of such an
iteration are fixed from step to step and can be recorded once and replayed."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_11530_amd import binding as pkv
from paper_2602_11530_amd import workloads as wl

from gpu_util import MAX_ABS, REL_L2, assert_launchable, run_attn_dev, shape_of, to_bits, to_dev

pytestmark = pytest.mark.gpu


def layer_tensors(w, rng):
    return (wl.normal_bf16(rng, w.q_shape()), wl.normal_bf16(rng, w.pool_shape()),
            wl.normal_bf16(rng, w.pool_shape()))


def check(got_bits, q, k, v, w, what):
    ref = oracle.paged_decode_attn(q, k, v, w.block_tables, w.context_lens, w.scale)
    c = oracle.compare(got_bits, ref)
    print(f"{what}: {c}", flush=True)
    assert c["max_abs"] <= MAX_ABS and c["rel_l2"] <= REL_L2, (what, c)


@pytest.mark.parametrize("P", [0, 64])
def test_layers_call_equals_single_calls(device, P):
    w = wl.custom([700, 17, 2049, 0, 1, 333, 1024, 96], 40, 8, seed=51, num_pool_blocks=400)
    assert_launchable(w)
    rng = np.random.default_rng(51)
    n_layers = 5
    host = [layer_tensors(w, rng) for _ in range(n_layers)]
    dev = [tuple(to_dev(x) for x in t) for t in host]
    t_d, l_d = to_dev(w.block_tables), to_dev(w.context_lens)
    single = [run_attn_dev(w, q, k, v, t_d, l_d, partition_size=P) for q, k, v in dev]
    shape = shape_of(w, P)
    ws = torch.empty(pkv.pkv_attn_workspace_bytes(shape), dtype=torch.uint8, device=device)
    outs = [torch.full(w.q_shape(), 0x7FC1, dtype=torch.int16, device=device) for _ in range(n_layers)]
    pkv.paged_decode_attn_layers([d[0] for d in dev], [d[1] for d in dev], [d[2] for d in dev],
                                 t_d, l_d, float(w.scale), outs, shape, ws)
    torch.cuda.synchronize()
    for l in range(n_layers):
        assert torch.equal(outs[l], single[l]), f"layer {l} differs from its single call"
        check(to_bits(outs[l]), *host[l], w, f"layers call P={P}, layer {l}")
    # zero layers and an empty batch launch nothing
    pkv.paged_decode_attn_layers([], [], [], t_d, l_d, float(w.scale), [], shape, ws)
    w0 = wl.custom([], 40, 8, seed=1, num_pool_blocks=4, maxb=4)
    pkv.paged_decode_attn_layers([dev[0][0]], [dev[0][1]], [dev[0][2]], None, None, 1.0,
                                 [outs[0]], shape_of(w0), None)
    torch.cuda.synchronize()
    assert torch.equal(outs[0], single[0])


def test_graph_replay_of_decode_steps(device):
    """kv_append + attention of three layers recorded once, replayed for four
    decode steps.  Between replays the host refreshes the static input buffers
    and the lengths grow by one on the device; every replay is compared with the
    same step run eagerly on copies of the pools and with the oracle."""
    n_layers, n_steps = 3, 4
    final = np.array([40, 16 * 9 + 1, 1030, 5, 2300, 64], np.int32)
    w = wl.custom(final, 40, 8, seed=57, num_pool_blocks=330)   # tables cover the final lengths
    rng = np.random.default_rng(57)
    host = [layer_tensors(w, rng) for _ in range(n_layers)]
    k_h = [h[1].copy() for h in host]
    v_h = [h[2].copy() for h in host]
    k_g = [to_dev(x) for x in k_h]      # pools the graph appends to
    v_g = [to_dev(x) for x in v_h]
    k_e = [x.clone() for x in k_g]      # pools the eager run appends to
    v_e = [x.clone() for x in v_g]
    t_d = to_dev(w.block_tables)
    shape = shape_of(w)                 # launch sized for the table's capacity: lengths may grow
    ws = torch.empty(pkv.pkv_attn_workspace_bytes(shape), dtype=torch.uint8, device=device)
    S, Hkv = w.num_seqs, w.num_kv_heads
    # static buffers: the graph always reads these addresses
    lens_d = to_dev(final - n_steps)
    q_s = [torch.zeros(w.q_shape(), dtype=torch.int16, device=device) for _ in range(n_layers)]
    kn_s = [torch.zeros((S, Hkv, 128), dtype=torch.int16, device=device) for _ in range(n_layers)]
    vn_s = [torch.zeros((S, Hkv, 128), dtype=torch.int16, device=device) for _ in range(n_layers)]
    out_s = [torch.full(w.q_shape(), 0x7FC1, dtype=torch.int16, device=device) for _ in range(n_layers)]

    def decode_step(k_pools, v_pools, outs):
        for l in range(n_layers):
            pkv.kv_append(kn_s[l], vn_s[l], k_pools[l], v_pools[l], t_d, lens_d, shape)
            pkv.paged_decode_attn(q_s[l], k_pools[l], v_pools[l], t_d, lens_d, float(w.scale),
                                  outs[l], shape, ws)

    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):       # binding calls enqueue on the capturing stream
        decode_step(k_g, v_g, out_s)
    torch.cuda.synchronize()
    # capture executes nothing
    assert all(torch.equal(a, b) for a, b in zip(k_g, k_e))

    for step in range(n_steps):
        lens_d.add_(1)
        w.context_lens = final - n_steps + step + 1
        assert_launchable(w)
        new = []
        for l in range(n_layers):
            q = wl.normal_bf16(rng, w.q_shape())
            kn = wl.normal_bf16(rng, (S, Hkv, 128))
            vn = wl.normal_bf16(rng, (S, Hkv, 128))
            q_s[l].copy_(to_dev(q)); kn_s[l].copy_(to_dev(kn)); vn_s[l].copy_(to_dev(vn))
            new.append((q, kn, vn))
        for o in out_s:
            o.fill_(0x7FC1)
        graph.replay()
        torch.cuda.synchronize()
        replayed = [o.clone() for o in out_s]
        eager = [torch.full(w.q_shape(), 0x7FC1, dtype=torch.int16, device=device) for _ in range(n_layers)]
        decode_step(k_e, v_e, eager)
        torch.cuda.synchronize()
        for l in range(n_layers):
            assert torch.equal(replayed[l], eager[l]), f"step {step} layer {l}: replay != eager"
            assert torch.equal(k_g[l], k_e[l]) and torch.equal(v_g[l], v_e[l]), f"step {step} layer {l}: pools"
            q, kn, vn = new[l]
            k_h[l], v_h[l] = oracle.kv_append(kn, vn, k_h[l], v_h[l], w.block_tables, w.context_lens)
            assert np.array_equal(to_bits(k_g[l]).reshape(k_h[l].shape), k_h[l])
            check(to_bits(replayed[l]), q, k_h[l], v_h[l], w, f"graph replay step {step} layer {l}")


def test_two_instances_decode_concurrently(device):
    """Two instances on the one GPU, each with its own pools, tables, workspace and stream:
    their attention calls may overlap in time and must not disturb each other."""
    rng = np.random.default_rng(71)
    ws_ = [wl.custom(rng.integers(200, 3000, size=12), 40, 8, seed=71 + i) for i in range(2)]
    host = [wl.make_host_tensors(w) for w in ws_]
    dev = [tuple(to_dev(x) for x in h) for h in host]
    tabs = [(to_dev(w.block_tables), to_dev(w.context_lens)) for w in ws_]
    alone = [run_attn_dev(w, *d, *t) for w, d, t in zip(ws_, dev, tabs)]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(device), torch.cuda.Stream(device)]
    shapes = [shape_of(w) for w in ws_]
    wss = [torch.empty(pkv.pkv_attn_workspace_bytes(s), dtype=torch.uint8, device=device) for s in shapes]
    outs = [torch.full(w.q_shape(), 0x7FC1, dtype=torch.int16, device=device) for w in ws_]
    torch.cuda.synchronize()   # the fills ran on the default stream; the side streams do not wait for it
    for rep in range(6):
        for i in (0, 1):
            q, k, v = dev[i]
            pkv.paged_decode_attn(q, k, v, tabs[i][0], tabs[i][1], float(ws_[i].scale), outs[i],
                                  shapes[i], wss[i], streams[i])
    torch.cuda.synchronize()
    for i in (0, 1):
        assert torch.equal(outs[i], alone[i]), f"instance {i} changed when run next to the other"
        check(to_bits(outs[i]), *host[i], ws_[i], f"concurrent instance {i}")
