#!/usr/bin/env python3
"""Benchmark of the paged-decode hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic batch:
  1. paged_decode_attn over every request of the batch (block-table staging,
     QK, online softmax, PV, partition epilogue, split-K reduce), then
  2. a migration of a seeded 25 % of the requests: kv_blocks_gather of their K
     and V blocks into a staging buffer and kv_blocks_scatter into reshuffled
     block ids.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E bandwidth

# HBM bytes per launch of the stream kernel from rocprofv3 FETCH_SIZE + WRITE_SIZE, each scaled by
# what the same counter reads for the copy kernel of known size (profiles/attn_stream_cfg2.md,
# profiles/attn_stream_cfg3.md); quoted only for the partitioning those profiles were taken with.
MEASURED_TRAFFIC_BYTES = {"cfg2_qwen32b_b64_u1024_8192": 1219560000,
                          "cfg3_longcot_b128_lognormal": 4110160000}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg4"],
                    help="cfg4: the full-depth phase-mixed batch, every layer's pools resident, one "
                         "multi-layer attention call per step (no migration; use --steps 5)")
    ap.add_argument("--layers", type=int, default=0, help="cfg4 only: layers to keep resident (0 = 64, or what fits)")
    ap.add_argument("--partition", type=int, default=None,
                    help="split-K partition in tokens (default: the workload's; 0 = library picks)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-migration", action="store_true",
                    help="time the attention call alone (profiling aid; not the headline step)")
    return ap.parse_args()


def device_tensors(w, device):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(w.seed + 17)
    q = torch.randn(w.q_shape(), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    pools = []
    for _ in range(2):
        p = torch.empty(w.pool_shape(), dtype=torch.bfloat16, device=device)
        flat = p.view(-1)
        step = 1 << 28
        for o in range(0, flat.numel(), step):
            n = min(step, flat.numel() - o)
            flat[o:o + n] = torch.randn(n, generator=g, device=device, dtype=torch.float32)
        pools.append(p)
    return q, pools[0], pools[1]


def full_depth(args, dev):
    """Config 4: 96 requests (70 % reasoning, 30 % answering lengths), one K and one V pool per
    layer, all resident; a step is one decode iteration's attention in every layer."""
    import numpy as np
    import torch

    from paper_2602_11530_amd import binding as pkv
    from paper_2602_11530_amd import workloads as wl

    w = wl.cfg4_phase_mixed()
    free, _ = torch.cuda.mem_get_info(dev)
    per_layer = 2 * w.num_pool_blocks * w.block_bytes + (4 << 20)
    n_layers = max(1, min(args.layers or w.num_layers, int((free - (24 << 30)) // per_layer)))
    g = torch.Generator(device=dev)
    layers = []
    for l in range(n_layers):
        g.manual_seed(w.seed + 1000 * l + 17)
        q = torch.randn(w.q_shape(), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
        pools = []
        for _ in range(2):
            p = torch.empty(w.pool_shape(), dtype=torch.bfloat16, device=dev)
            flat = p.view(-1)
            for o in range(0, flat.numel(), 1 << 28):
                n = min(1 << 28, flat.numel() - o)
                flat[o:o + n] = torch.randn(n, generator=g, device=dev, dtype=torch.float32)
            pools.append(p)
        layers.append((q, pools[0], pools[1]))
    outs = [torch.empty(w.q_shape(), dtype=torch.bfloat16, device=dev) for _ in range(n_layers)]
    tables = torch.from_numpy(w.block_tables).to(dev)
    lens = torch.from_numpy(w.context_lens).to(dev)
    shape = pkv.make_shape(w.num_seqs, w.num_q_heads, w.num_kv_heads, w.max_blocks_per_seq,
                           w.num_pool_blocks, max_context_len=int(w.context_lens.max()))
    ws = torch.empty(pkv.pkv_attn_workspace_bytes(shape), dtype=torch.uint8, device=dev)
    ptrs = [pkv.pointer_array(x) for x in ([l[0] for l in layers], [l[1] for l in layers],
                                           [l[2] for l in layers], outs)]
    stream = torch.cuda.current_stream()

    def step():
        pkv.paged_decode_attn_layers(ptrs[0], ptrs[1], ptrs[2], tables, lens, float(w.scale), ptrs[3],
                                     shape, ws, stream)

    for _ in range(max(1, min(args.warmup, 3))):
        step()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record(stream)
        step()
        b.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = np.array([a.elapsed_time(b) for a, b in ev])
    step_bytes = w.attn_algorithmic_bytes() * n_layers
    value = step_bytes / (wall / args.steps) / 1e9
    gbps = step_bytes / (ms.mean() * 1e-3) / 1e9
    res = {
        "metric": "paged decode attn HBM GB/s (% of peak) + KV tokens attended/s, Qwen-32B shape",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": max(1, min(args.warmup, 3)), "ms_per_step": round(wall * 1e3 / args.steps, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "num_seqs": w.num_seqs, "q_heads": w.num_q_heads,
                   "kv_heads": w.num_kv_heads, "layers_resident": n_layers,
                   "resident_kv_bytes": n_layers * 2 * w.num_pool_blocks * w.block_bytes,
                   "total_context_tokens": w.total_tokens,
                   "step": "paged_decode_attn_layers over every resident layer"},
        "step_algorithmic_bytes": step_bytes,
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "attn": {"ms_mean": round(float(ms.mean()), 3), "GBps": round(gbps, 1),
                 "kv_tokens_attended_per_s": round(w.total_tokens * n_layers / (ms.mean() * 1e-3), 1),
                 "token_definition": "one cached position of one request attended in one layer by all its heads"},
        "roofline": {"bound": "hbm", "kernel": "attn_stream_kernel + merge, all layers of a step",
                     "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": None},
        "cpu_baseline": None,
    }
    print(json.dumps(res), flush=True)


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the path shards by request or by KV head with no exchange inside the call).",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2602_11530_amd import binding as pkv
    from paper_2602_11530_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.workload == "cfg4":
        return full_depth(args, dev)
    w = {"cfg1": wl.cfg1_tiny, "cfg2": wl.cfg2_qwen32b, "cfg3": wl.cfg3_long_cot}[args.workload]()
    if args.partition is not None:
        w.partition_size = args.partition
    q, k_pool, v_pool = device_tensors(w, dev)
    tables = torch.from_numpy(w.block_tables).to(dev)
    lens = torch.from_numpy(w.context_lens).to(dev)
    out = torch.empty(w.q_shape(), dtype=torch.bfloat16, device=dev)
    max_ctx = int(w.context_lens.max())
    shape = pkv.make_shape(w.num_seqs, w.num_q_heads, w.num_kv_heads, w.max_blocks_per_seq,
                           w.num_pool_blocks, partition_size=w.partition_size,
                           max_context_len=max_ctx)
    P = pkv.pkv_attn_partition_size(shape)
    ws_bytes = pkv.pkv_attn_workspace_bytes(shape)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    mig = wl.make_migration(w, 0.25)
    n_mig = 0 if args.no_migration else len(mig.old_ids)
    old_ids = torch.from_numpy(mig.old_ids).to(dev)
    new_ids = torch.from_numpy(mig.new_ids).to(dev)
    staging = torch.empty((max(n_mig, 1),) + tuple(w.pool_shape()[1:]), dtype=torch.bfloat16,
                          device=dev)
    scale = float(w.scale)
    stream = torch.cuda.current_stream()
    bb, NB = w.block_bytes, w.num_pool_blocks

    # The migration permutes rows among the victims' blocks, so the attention
    # of later steps reads the same bytes in another order: same traffic.
    def step(ev=None):
        if ev is not None:
            ev[0].record(stream)
        pkv.paged_decode_attn(q, k_pool, v_pool, tables, lens, scale, out, shape, ws, stream)
        if ev is not None:
            ev[1].record(stream)
        if n_mig:
            pkv.kv_blocks_gather(k_pool, old_ids, staging, n_mig, bb, NB, stream)
            pkv.kv_blocks_scatter(staging, k_pool, new_ids, n_mig, bb, NB, stream)
            pkv.kv_blocks_gather(v_pool, old_ids, staging, n_mig, bb, NB, stream)
            pkv.kv_blocks_scatter(staging, v_pool, new_ids, n_mig, bb, NB, stream)
        if ev is not None:
            ev[2].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_step = wall * 1e3 / args.steps
    attn_ms = np.array([e[0].elapsed_time(e[1]) for e in events])
    mig_ms = np.array([e[1].elapsed_time(e[2]) for e in events])
    attn_bytes = w.attn_algorithmic_bytes()
    # each migrated block is read once and written once by the gather and again by the scatter
    mig_bytes = 2 * (2 * 2 * n_mig * bb + 2 * 4 * n_mig)
    step_bytes = attn_bytes + mig_bytes
    value = step_bytes / (ms_step * 1e-3) / 1e9
    attn_gbps = attn_bytes / (attn_ms.mean() * 1e-3) / 1e9
    tokens_per_s = w.total_tokens / (attn_ms.mean() * 1e-3)

    res = {
        "metric": "paged decode attn HBM GB/s (% of peak) + KV tokens attended/s, Qwen-32B shape",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": w.name,
            "num_seqs": w.num_seqs, "q_heads": w.num_q_heads, "kv_heads": w.num_kv_heads,
            "head_dim": w.head_dim, "block_size": w.block_size,
            "total_context_tokens": w.total_tokens, "pool_blocks": w.num_pool_blocks,
            "partition_size": P, "migrated_blocks_per_pool": n_mig,
            "step": "paged_decode_attn + gather/scatter of 25% of requests (K and V pools)"
                    if n_mig else "paged_decode_attn only",
        },
        "step_algorithmic_bytes": step_bytes,
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "attn": {
            "algorithmic_bytes": attn_bytes,
            "ms_mean": round(float(attn_ms.mean()), 4), "ms_median": round(float(np.median(attn_ms)), 4),
            "ms_min": round(float(attn_ms.min()), 4),
            "GBps": round(attn_gbps, 1), "pct_of_hbm_peak": round(100 * attn_gbps / HBM_PEAK_GBPS, 2),
            "kv_tokens_attended_per_s": round(tokens_per_s, 1),
            "token_definition": "one cached position of one request attended in one layer by all its heads",
            "workspace_bytes": ws_bytes,
        },
        "migration": None if not n_mig else {
            "algorithmic_bytes": mig_bytes, "ms_mean": round(float(mig_ms.mean()), 4),
            "GBps_read_plus_write": round(mig_bytes / (mig_ms.mean() * 1e-3) / 1e9, 1),
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "attn_stream_kernel (event-timed together with the small merge kernel that follows it)",
            "achieved": round(attn_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(attn_gbps / HBM_PEAK_GBPS, 4),
            "traffic": MEASURED_TRAFFIC_BYTES.get(w.name) if args.partition is None else None,
        },
    }

    if not args.no_cpu_baseline:
        import oracle
        qh = q.view(torch.int16).cpu().numpy().view(np.uint16)
        kh = k_pool.view(torch.int16).cpu().numpy().view(np.uint16)
        vh = v_pool.view(torch.int16).cpu().numpy().view(np.uint16)
        ref, secs, threads = oracle.timed_attn(qh, kh, vh, w.block_tables, w.context_lens, w.scale)
        # The pools were copied after the timed loop; one more step attends over
        # exactly that state (its migration runs after its attention).
        step()
        torch.cuda.synchronize()
        got = out.view(torch.int16).cpu().numpy().view(np.uint16)
        cmp_ = oracle.compare(got, ref)
        res["cpu_baseline"] = {
            "value": round(attn_bytes / secs / 1e9, 3), "unit": "GB/s", "cores": threads,
            "kind": "oracle",
            "sample": f"the whole attention call of {w.name} ({w.num_seqs} requests, "
                      f"{w.total_tokens} context tokens), {secs:.2f} s; migration not included",
            "kv_tokens_attended_per_s": round(w.total_tokens / secs, 1),
        }
        res["parity"] = {k: float(f"{v:.3e}") for k, v in cmp_.items()}
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
