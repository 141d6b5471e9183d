#!/usr/bin/env python3
"""Benchmark of the paged-decode hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic batch:
  1. paged_decode_attn over every request of the batch (block-table staging,
     QK, online softmax, PV, partition epilogue, split-K reduce), then
  2. a migration of a seeded 25 % of the requests: kv_blocks_gather of their K
     and V blocks into a staging buffer and kv_blocks_scatter into reshuffled
     block ids.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

The default run times the Qwen-32B-shaped batch the metric is quoted on and,
in the same line under "cfg3", the long-context batch at its specified
512-token partitions.  Other modes: --workload cfg3 | cfg4 | cfg5 | cfg1;
--kv-dtype fp8 (8-bit pools), --head-dim 64|256, --batch N and
--context-range LO HI (config 2's shape at other sizes), each a workload of its
own, named as such.  Next to the attention rate the line carries what this box
delivers for the same access pattern with no arithmetic (box_stream_read) and
for a plain device-to-device copy (box_copy_bandwidth).
`--record-traffic` (no GPU) turns two rocprofv3 counter runs of this script
into profiles/hbm_traffic.json, which later runs quote as roofline.traffic.
"""
from __future__ import annotations

import argparse
import csv
import hashlib
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E bandwidth
METRIC = "paged decode attn HBM GB/s (% of peak) + KV tokens attended/s, Qwen-32B shape"
TOKEN_DEF = "one cached position of one request attended in one layer by all its heads"
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
KERNEL_SOURCES = ["attn_stream.hip", "attn_reduce.hip", "pkv_kernels.h"]
MAX_ABS, REL_L2 = 1e-2, 5e-3


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"],
                    help="cfg2 (default) also reports cfg3 in a sub-record; cfg4: the full-depth batch, "
                         "every layer's pools resident, one multi-layer attention call per step (use "
                         "--steps 5); cfg5: migration of 25 %% of cfg4's requests next to decode of the rest")
    ap.add_argument("--layers", type=int, default=0, help="cfg4/cfg5: layers to keep resident (0 = 64, or what fits)")
    ap.add_argument("--partition", type=int, default=None,
                    help="split-K partition in tokens (default: the workload's; 0 = library picks)")
    ap.add_argument("--migrate-fraction", type=float, default=0.25,
                    help="fraction of the requests whose blocks the step migrates (default 0.25)")
    ap.add_argument("--kv-dtype", default="bf16", choices=["bf16", "fp8"],
                    help="fp8: the same batch with one-byte E4M3 KV pools (cfg2/cfg3; a workload of its "
                         "own, reported as such)")
    ap.add_argument("--head-dim", type=int, default=128, choices=[64, 128, 256],
                    help="cfg2 only: the same batch at another head dimension (a workload of its own, "
                         "named ..._d64 / ..._d256)")
    ap.add_argument("--batch", type=int, default=64,
                    help="cfg2 only: number of requests (another workload, named for its sizes)")
    ap.add_argument("--context-range", type=int, nargs=2, default=[1024, 8192], metavar=("LO", "HI"),
                    help="cfg2 only: context lengths are drawn from U{LO..HI}")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cfg3", action="store_true", help="default run: skip the long-context sub-record")
    ap.add_argument("--no-migration", action="store_true",
                    help="time the attention call alone (profiling aid; not the headline step)")
    ap.add_argument("--record-traffic", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="no GPU: read the counter_collection csv files of two `rocprofv3 --pmc FETCH_SIZE` / "
                         "`--pmc WRITE_SIZE` runs of this script on --workload and update profiles/hbm_traffic.json")
    return ap.parse_args()


# ---------------------------------------------------------------------------
# HBM traffic measured with rocprofv3 counters, kept in a tracked file
# ---------------------------------------------------------------------------
def kernel_sources_digest() -> str:
    """Identifies the kernels a traffic figure was measured on: the sources and the build flags."""
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        h.update(open(os.path.join(ROOT, "paper_2602_11530_amd", "csrc", name), "rb").read())
    from paper_2602_11530_amd import build as pkv_build
    h.update(" ".join(pkv_build.FLAGS).encode())
    return h.hexdigest()


def recorded_traffic(workload_name: str, partition: int):
    """Bytes per attention launch from the tracked counter file, or None when the file was
    measured on other kernels, another partitioning or another workload."""
    try:
        rec = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        return None
    if rec.get("kernel_sources_sha256") != kernel_sources_digest():
        return None
    w = rec.get("workloads", {}).get(workload_name)
    if not w or w.get("partition_size") != partition:
        return None
    return w["attn_stream_bytes_per_launch"]


def record_traffic(args):
    """profiles/hbm_traffic.json from two counter runs.  Each counter is scaled by what it reads
    for the gather kernel, which reads and writes exactly n_blocks * block_bytes."""
    from paper_2602_11530_amd import workloads as wl
    w = {"cfg2": wl.cfg2_qwen32b, "cfg3": wl.cfg3_long_cot}[args.workload]()
    mig = wl.make_migration(w, args.migrate_fraction)
    known_kib = len(mig.old_ids) * w.block_bytes / 1024.0

    def per_kernel(path, counter):
        acc = {}
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] != counter:
                continue
            acc.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
        return {k: sum(v) / len(v) for k, v in acc.items()}

    out = {}
    for path, counter, key in ((args.record_traffic[0], "FETCH_SIZE", "fetch"),
                               (args.record_traffic[1], "WRITE_SIZE", "write")):
        k = per_kernel(path, counter)
        gather = [v for n, v in k.items() if "kv_block_copy_kernel<0" in n]
        stream = [v for n, v in k.items() if "attn_stream_kernel" in n]
        if len(gather) != 1 or len(stream) != 1:
            sys.exit(f"{path}: expected one gather and one stream kernel, found {sorted(k)}")
        scale = known_kib / gather[0]
        out[key + "_counter_per_KiB"] = gather[0] / known_kib
        out[key + "_bytes"] = int(round(stream[0] * scale * 1024))
    P = args.partition if args.partition is not None else w.partition_size
    try:
        rec = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        rec = {}
    digest = kernel_sources_digest()
    if rec.get("kernel_sources_sha256") != digest:
        rec = {"kernel_sources_sha256": digest, "workloads": {}}
    try:   # the commit whose tree holds the measured kernel sources: HEAD, unless they are modified
        dirty = subprocess.run(["git", "-C", ROOT, "diff", "--quiet", "HEAD", "--"] +
                               [os.path.join("paper_2602_11530_amd", "csrc", n) for n in KERNEL_SOURCES]).returncode
        head = subprocess.check_output(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], text=True).strip()
        rec["commit"] = head + (" + uncommitted changes to the kernel sources" if dirty else "")
    except (OSError, subprocess.CalledProcessError):
        rec["commit"] = None
    rec["note"] = ("rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (KiB per dispatch), averaged over the "
                   "dispatches of attn_stream_kernel, each scaled by the same counter's reading for the "
                   "gather kernel of known size; valid for the kernel sources with this digest only")
    from paper_2602_11530_amd import binding as pkv
    shape = pkv.make_shape(w.num_seqs, w.num_q_heads, w.num_kv_heads, w.max_blocks_per_seq,
                           w.num_pool_blocks, partition_size=P)
    rec["workloads"][w.name] = {
        "partition_size": pkv.pkv_attn_partition_size(shape),
        "algorithmic_bytes": w.attn_algorithmic_bytes(),
        "attn_stream_bytes_per_launch": out["fetch_bytes"] + out["write_bytes"],
        **out,
    }
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(rec, f, indent=1, sort_keys=True)
        f.write("\n")
    print(json.dumps(rec["workloads"][w.name]))


# ---------------------------------------------------------------------------
# helpers
# ---------------------------------------------------------------------------
def fill_layer(w, seed, dev):
    """Seeded N(0,1) bf16 q, K pool and V pool made on the device."""
    import torch
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    q = torch.randn(w.q_shape(), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    pools = []
    for _ in range(2):
        p = torch.empty(w.pool_shape(), dtype=torch.bfloat16, device=dev)
        flat = p.view(-1)
        for o in range(0, flat.numel(), 1 << 28):
            n = min(1 << 28, flat.numel() - o)
            flat[o:o + n] = torch.randn(n, generator=g, device=dev, dtype=torch.float32)
        pools.append(p)
    return q, pools[0], pools[1]


KV_SCALES = (0.0134, 0.0171)   # E4M3 pools: 448 * scale covers 6 and 7.7 sigma of the N(0,1) rows


def fill_layer_fp8(w, seed, dev):
    """q in bf16; K and V pools as E4M3 bytes whose de-quantised values are ~N(0,1)."""
    import torch
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    q = torch.randn(w.q_shape(), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    pools = []
    for scale in KV_SCALES:
        p = torch.empty(w.pool_shape(), dtype=torch.uint8, device=dev)
        flat = p.view(-1)
        for o in range(0, flat.numel(), 1 << 28):
            n = min(1 << 28, flat.numel() - o)
            x = torch.randn(n, generator=g, device=dev, dtype=torch.float32) / scale
            flat[o:o + n] = x.clamp_(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8)
        pools.append(p)
    return q, pools[0], pools[1]


def box_copy_bandwidth(dev):
    """Read+write GB/s of a plain device-to-device copy of 1 GiB on this machine (the practical
    ceiling for mixed traffic, reported next to the nominal peak)."""
    import torch
    n = 1 << 30
    a = torch.empty(n, dtype=torch.uint8, device=dev)
    b = torch.empty(n, dtype=torch.uint8, device=dev)
    a.fill_(1)
    for _ in range(2):
        b.copy_(a)
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for _ in range(10):
        b.copy_(a)
    t1.record()
    torch.cuda.synchronize()
    return 10 * 2 * n / (t0.elapsed_time(t1) * 1e-3) / 1e9


def base_line(args, value, ms_per_step, steps, warmup):
    return {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
    }


# ---------------------------------------------------------------------------
# one layer: attention + migration (cfg1, cfg2, cfg3)
# ---------------------------------------------------------------------------
def single_layer(args, w, dev, steps, warmup, cpu_baseline):
    import numpy as np
    import torch

    from paper_2602_11530_amd import binding as pkv
    from paper_2602_11530_amd import workloads as wl

    fp8 = args.kv_dtype == "fp8"
    q, k_pool, v_pool = (fill_layer_fp8 if fp8 else fill_layer)(w, w.seed + 17, dev)
    elem = 1 if fp8 else 2
    tables = torch.from_numpy(w.block_tables).to(dev)
    lens = torch.from_numpy(w.context_lens).to(dev)
    out = torch.empty(w.q_shape(), dtype=torch.bfloat16, device=dev)
    max_ctx = int(w.context_lens.max())
    shape = pkv.make_shape(w.num_seqs, w.num_q_heads, w.num_kv_heads, w.max_blocks_per_seq,
                           w.num_pool_blocks, head_dim=w.head_dim, block_size=w.block_size,
                           partition_size=w.partition_size, max_context_len=max_ctx)
    P = pkv.pkv_attn_partition_size(shape)
    ws_bytes = pkv.pkv_attn_workspace_bytes(shape)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    mig = wl.make_migration(w, args.migrate_fraction)
    n_mig = 0 if args.no_migration else len(mig.old_ids)
    old_ids = torch.from_numpy(mig.old_ids).to(dev)
    new_ids = torch.from_numpy(mig.new_ids).to(dev)
    staging = torch.empty((max(n_mig, 1),) + tuple(w.pool_shape()[1:]), dtype=k_pool.dtype,
                          device=dev)
    scale = float(w.scale)
    stream = torch.cuda.current_stream()
    bb, NB = w.block_bytes * elem // 2, w.num_pool_blocks

    def attention():
        if fp8:
            pkv.paged_decode_attn_fp8kv(q, k_pool, v_pool, tables, lens, scale, KV_SCALES[0],
                                        KV_SCALES[1], out, shape, ws, stream)
        else:
            pkv.paged_decode_attn(q, k_pool, v_pool, tables, lens, scale, out, shape, ws, stream)

    # The migration permutes rows among the victims' blocks, so the attention
    # of later steps reads the same bytes in another order: same traffic.
    def step(ev=None):
        if ev is not None:
            ev[0].record(stream)
        attention()
        if ev is not None:
            ev[1].record(stream)
        if n_mig:
            pkv.kv_blocks_gather(k_pool, old_ids, staging, n_mig, bb, NB, stream)
            pkv.kv_blocks_scatter(staging, k_pool, new_ids, n_mig, bb, NB, stream)
            pkv.kv_blocks_gather(v_pool, old_ids, staging, n_mig, bb, NB, stream)
            pkv.kv_blocks_scatter(staging, v_pool, new_ids, n_mig, bb, NB, stream)
        if ev is not None:
            ev[2].record(stream)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_step = wall * 1e3 / steps
    attn_ms = np.array([e[0].elapsed_time(e[1]) for e in events])
    mig_ms = np.array([e[1].elapsed_time(e[2]) for e in events])
    # every valid K and V row once (at one or two bytes per element), q, out, tables, lengths
    attn_bytes = w.attn_algorithmic_bytes() - (2 - elem) * w.total_tokens * w.num_kv_heads * w.head_dim * 2
    # each migrated block is read once and written once by the gather and again by the scatter
    mig_bytes = 2 * (2 * 2 * n_mig * bb + 2 * 4 * n_mig)
    step_bytes = attn_bytes + mig_bytes
    attn_gbps = attn_bytes / (attn_ms.mean() * 1e-3) / 1e9

    res = {
        "ms_per_step": ms_step,
        "config": {
            "workload": w.name + ("_fp8kv" if fp8 else ""),
            "kv_dtype": "e4m3 bytes, one fp32 scale per pool" if fp8 else "bf16",
            "num_seqs": w.num_seqs, "q_heads": w.num_q_heads, "kv_heads": w.num_kv_heads,
            "head_dim": w.head_dim, "block_size": w.block_size,
            "total_context_tokens": w.total_tokens, "pool_blocks": w.num_pool_blocks,
            "partition_size": P, "migrated_blocks_per_pool": n_mig,
            "step": "paged_decode_attn + gather/scatter of 25% of requests (K and V pools)"
                    if n_mig else "paged_decode_attn only",
        },
        "attn": {
            "algorithmic_bytes": attn_bytes,
            "ms_mean": round(float(attn_ms.mean()), 4), "ms_median": round(float(np.median(attn_ms)), 4),
            "ms_min": round(float(attn_ms.min()), 4),
            "GBps": round(attn_gbps, 1), "pct_of_hbm_peak": round(100 * attn_gbps / HBM_PEAK_GBPS, 2),
            "kv_tokens_attended_per_s": round(w.total_tokens / (attn_ms.mean() * 1e-3), 1),
            "token_definition": TOKEN_DEF,
            "workspace_bytes": ws_bytes,
        },
        "migration": None if not n_mig else {
            "algorithmic_bytes": mig_bytes, "staging_bytes": n_mig * bb,
            "ms_mean": round(float(mig_ms.mean()), 4),
            "GBps_read_plus_write": round(mig_bytes / (mig_ms.mean() * 1e-3) / 1e9, 1),
        },
        "step": {
            "algorithmic_bytes": step_bytes, "ms": round(ms_step, 4),
            "GBps": round(step_bytes / (ms_step * 1e-3) / 1e9, 1),
            "pct_of_hbm_peak": round(100 * step_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2),
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "attn_stream_kernel (event-timed together with the small merge kernel that follows it)",
            "achieved": round(attn_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(attn_gbps / HBM_PEAK_GBPS, 4),
            "traffic": None if fp8 else recorded_traffic(w.name, P),
        },
        "cpu_baseline": None,
    }

    if not fp8 and w.head_dim == 128:
        # What this box allows for the stream pass's own access pattern (same launch shape and
        # load instructions over hashed slabs of these pools, no arithmetic): pkv_probe_stream_read.
        units = int(((w.context_lens.astype(np.int64) + 15) // 16).sum()) * w.num_kv_heads
        slabs = w.num_pool_blocks * w.num_kv_heads * (w.block_size // 16)
        for _ in range(5):
            pkv.pkv_probe_stream_read(k_pool, v_pool, slabs, units, None, stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(50):
            pkv.pkv_probe_stream_read(k_pool, v_pool, slabs, units, None, stream)
        e1.record(stream)
        torch.cuda.synchronize()
        probe_ms = e0.elapsed_time(e1) / 50
        probe_gbps = units * 8192 / (probe_ms * 1e-3) / 1e9
        res["box_stream_read"] = {
            "GBps": round(probe_gbps, 1), "ms": round(probe_ms, 4), "bytes": units * 8192,
            "what": "pkv_probe_stream_read over this batch's block count: the stream pass's launch shape "
                    "and loads on hashed 4 KiB slabs of the same pools, no arithmetic, timed in this run",
            "attn_pct_of_it": round(100 * attn_gbps / probe_gbps, 1),
        }

    if cpu_baseline:
        import oracle
        qh = q.view(torch.int16).cpu().numpy().view(np.uint16)
        if fp8:
            kh, vh = k_pool.cpu().numpy(), v_pool.cpu().numpy()
            t0 = time.perf_counter()
            ref = oracle.paged_decode_attn_fp8kv(qh, kh, vh, w.block_tables, w.context_lens, w.scale,
                                                 KV_SCALES[0], KV_SCALES[1])
            secs, threads = time.perf_counter() - t0, oracle.max_threads()
        else:
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
        res["parity"]["within_bar"] = bool(cmp_["max_abs"] <= MAX_ABS and cmp_["rel_l2"] <= REL_L2)
    del q, k_pool, v_pool, staging, ws
    torch.cuda.empty_cache()
    return res


# ---------------------------------------------------------------------------
# all layers resident: cfg4 (attention of a full-depth step) and cfg5 (migration next to decode)
# ---------------------------------------------------------------------------
def resident_layers(args, w, dev, extra_bytes=0):
    import torch
    free, _ = torch.cuda.mem_get_info(dev)
    per_layer = 2 * w.num_pool_blocks * w.block_bytes + (4 << 20)
    n_layers = max(1, min(args.layers or w.num_layers,
                          int((free - (24 << 30) - extra_bytes) // per_layer)))
    return n_layers, [fill_layer(w, w.seed + 1000 * l + 17, dev) for l in range(n_layers)]


def full_depth(args, dev):
    """Config 4: 96 requests (70 % reasoning, 30 % answering lengths), one K and one V pool per
    layer, all resident; a step is one decode iteration's attention in every layer."""
    import numpy as np
    import torch

    from paper_2602_11530_amd import binding as pkv
    from paper_2602_11530_amd import workloads as wl

    w = wl.cfg4_phase_mixed()
    n_layers, layers = resident_layers(args, w, dev)
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

    warmup = max(1, min(args.warmup, 3))
    for _ in range(warmup):
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
    res = base_line(args, value, wall * 1e3 / args.steps, args.steps, warmup)
    res.update({
        "config": {"workload": w.name, "num_seqs": w.num_seqs, "q_heads": w.num_q_heads,
                   "kv_heads": w.num_kv_heads, "layers_resident": n_layers,
                   "resident_kv_bytes": n_layers * 2 * w.num_pool_blocks * w.block_bytes,
                   "total_context_tokens": w.total_tokens,
                   "step": "paged_decode_attn_layers over every resident layer"},
        "step_algorithmic_bytes": step_bytes,
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "attn": {"ms_mean": round(float(ms.mean()), 3), "GBps": round(gbps, 1),
                 "kv_tokens_attended_per_s": round(w.total_tokens * n_layers / (ms.mean() * 1e-3), 1),
                 "token_definition": TOKEN_DEF},
        "roofline": {"bound": "hbm", "kernel": "attn_stream_kernel + merge, all layers of a step",
                     "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": None},
        "cpu_baseline": None,
    })
    print(json.dumps(res), flush=True)


def migration_next_to_decode(args, dev):
    """Config 5: 24 of config 4's 96 requests are migrated, layer by layer through one reused
    staging buffer (gather K, scatter K, gather V, scatter V), while a second stream decodes the
    72 survivors.  Reports the copies alone, the survivors' attention alone, and both together."""
    import numpy as np
    import torch

    from paper_2602_11530_amd import binding as pkv
    from paper_2602_11530_amd import workloads as wl

    w = wl.cfg4_phase_mixed()
    mig = wl.make_migration(w, 0.25)
    n = len(mig.old_ids)
    bb, NB = w.block_bytes, w.num_pool_blocks
    n_layers, layers = resident_layers(args, w, dev, extra_bytes=2 * n * bb)
    ws_surv = wl.subset(w, mig.survivors)
    surv_idx = torch.from_numpy(mig.survivors.astype(np.int64)).to(dev)
    q_surv = [q.index_select(0, surv_idx).contiguous() for q, _, _ in layers]
    outs = [torch.empty(ws_surv.q_shape(), dtype=torch.bfloat16, device=dev) for _ in range(n_layers)]
    tables = torch.from_numpy(ws_surv.block_tables).to(dev)
    lens = torch.from_numpy(ws_surv.context_lens).to(dev)
    shape = pkv.make_shape(ws_surv.num_seqs, w.num_q_heads, w.num_kv_heads, w.max_blocks_per_seq,
                           NB, max_context_len=int(ws_surv.context_lens.max()))
    ws = torch.empty(pkv.pkv_attn_workspace_bytes(shape), dtype=torch.uint8, device=dev)
    ptrs = [pkv.pointer_array(x) for x in (q_surv, [l[1] for l in layers], [l[2] for l in layers], outs)]
    old_d = torch.from_numpy(mig.old_ids).to(dev)
    new_d = torch.from_numpy(mig.new_ids).to(dev)
    staging = torch.empty((n,) + tuple(w.pool_shape()[1:]), dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()
    s_copy, s_attn = torch.cuda.Stream(dev), torch.cuda.Stream(dev)

    def copies():
        for _, k, v in layers:
            for pool in (k, v):
                pkv.kv_blocks_gather(pool, old_d, staging, n, bb, NB, s_copy)
                pkv.kv_blocks_scatter(staging, pool, new_d, n, bb, NB, s_copy)

    def attention():
        pkv.paged_decode_attn_layers(ptrs[0], ptrs[1], ptrs[2], tables, lens, float(w.scale), ptrs[3],
                                     shape, ws, s_attn)

    def timed(fns, reps):
        """Mean ms per repetition of each stream's work and of the whole; the streams' work is
        enqueued one after the other (the short enqueue first) and runs side by side."""
        per, whole = [[] for _ in fns], []
        for _ in range(reps):
            torch.cuda.synchronize()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in fns]
            t0 = time.perf_counter()
            for (fn, st), (a, b) in zip(fns, ev):
                a.record(st)
                fn()
                b.record(st)
            torch.cuda.synchronize()
            whole.append((time.perf_counter() - t0) * 1e3)
            for i, (a, b) in enumerate(ev):
                per[i].append(a.elapsed_time(b))
        return [float(np.mean(p)) for p in per], float(np.mean(whole))

    reps = max(1, args.steps)
    copies(); attention()                                   # warm-up
    (copy_ms,), _ = timed([(copies, s_copy)], reps)
    (attn_ms,), _ = timed([(attention, s_attn)], reps)
    (attn_c, copy_c), both_ms = timed([(attention, s_attn), (copies, s_copy)], reps)
    copy_bytes = n_layers * 2 * 2 * (2 * n * bb + 4 * n)     # 2 pools x (gather + scatter) x (read + write)
    attn_bytes = n_layers * ws_surv.attn_algorithmic_bytes()
    gb = lambda b, ms: round(b / (ms * 1e-3) / 1e9, 1)
    value = gb(copy_bytes + attn_bytes, both_ms)
    res = base_line(args, value, both_ms, reps, 1)
    res.update({
        "config": {"workload": "cfg5_migration_next_to_decode", "layers_resident": n_layers,
                   "victims": len(mig.victims), "survivors": len(mig.survivors),
                   "migrated_blocks_per_pool": n, "staging_bytes": n * bb,
                   "resident_kv_bytes": n_layers * 2 * NB * bb,
                   "step": "per layer gather+scatter of the victims' K and V blocks on one stream, "
                           "paged_decode_attn_layers of the survivors on another"},
        "copy_alone": {"ms": round(copy_ms, 3), "algorithmic_bytes": copy_bytes,
                       "GBps_read_plus_write": gb(copy_bytes, copy_ms),
                       "pct_of_hbm_peak": round(100 * gb(copy_bytes, copy_ms) / HBM_PEAK_GBPS, 2)},
        "attn_alone": {"ms": round(attn_ms, 3), "algorithmic_bytes": attn_bytes,
                       "GBps": gb(attn_bytes, attn_ms),
                       "pct_of_hbm_peak": round(100 * gb(attn_bytes, attn_ms) / HBM_PEAK_GBPS, 2),
                       "kv_tokens_attended_per_s": round(ws_surv.total_tokens * n_layers / (attn_ms * 1e-3), 1)},
        "concurrent": {"wall_ms": round(both_ms, 3), "copy_ms": round(copy_c, 3), "attn_ms": round(attn_c, 3),
                       "copy_GBps_read_plus_write": gb(copy_bytes, copy_c), "attn_GBps": gb(attn_bytes, attn_c),
                       "combined_GBps": value,
                       "copy_slowdown": round(copy_c / copy_ms, 3), "attn_slowdown": round(attn_c / attn_ms, 3),
                       "wall_vs_serial": round(both_ms / (copy_ms + attn_ms), 3)},
        "roofline": {"bound": "hbm", "kernel": "kv_block_copy_kernel (gather, scatter) next to attn_stream_kernel",
                     "achieved": value, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(value / HBM_PEAK_GBPS, 4), "traffic": None},
        "cpu_baseline": None,
    })
    print(json.dumps(res), flush=True)


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the path shards by request or by KV head with no exchange inside the call).",
              file=sys.stderr)
        sys.exit(2)
    if args.record_traffic:
        return record_traffic(args)

    import torch

    from paper_2602_11530_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.workload == "cfg4":
        return full_depth(args, dev)
    if args.workload == "cfg5":
        return migration_next_to_decode(args, dev)
    lo, hi = args.context_range
    resized = args.head_dim != 128 or args.batch != 64 or [lo, hi] != [1024, 8192]
    if resized and args.workload != "cfg2":
        print("bench.py: --head-dim, --batch and --context-range apply to --workload cfg2 only", file=sys.stderr)
        sys.exit(2)
    if not (1 <= args.batch <= 2048 and 1 <= lo <= hi):
        print("bench.py: --batch must be 1..2048 and --context-range 1 <= LO <= HI", file=sys.stderr)
        sys.exit(2)
    w = {"cfg1": wl.cfg1_tiny,
         "cfg2": lambda: wl.cfg2_qwen32b(batch=args.batch, lo=lo, hi=hi, head_dim=args.head_dim),
         "cfg3": wl.cfg3_long_cot}[args.workload]()
    if args.partition is not None:
        w.partition_size = args.partition
    r = single_layer(args, w, dev, args.steps, args.warmup, not args.no_cpu_baseline)
    # `value` is the metric's quantity: HBM GB/s of the attention call; the blended figure of the
    # whole step (attention + migration copies) is under "step"
    res = base_line(args, r["attn"]["GBps"], r["ms_per_step"], args.steps, args.warmup)
    if args.kv_dtype == "fp8":
        res["dtype"] = "bf16 arithmetic operands and output, e4m3 KV pools"
    res["pct_of_hbm_peak"] = r["attn"]["pct_of_hbm_peak"]
    res.update({k: v for k, v in r.items() if k != "ms_per_step"})
    copy_gbps = box_copy_bandwidth(dev)
    res["box_copy_bandwidth"] = {
        "GBps_read_plus_write": round(copy_gbps, 1),
        "what": "device-to-device copy of 1 GiB timed in this run",
        "attn_pct_of_it": round(100 * r["attn"]["GBps"] / copy_gbps, 1),
    }
    ok = r.get("parity", {}).get("within_bar", True)

    if args.workload == "cfg2" and not args.no_cfg3 and args.partition is None and args.kv_dtype == "bf16" \
            and not resized:
        # The long-context batch as specified (512-token partitions), in the same line.  It is
        # measured by a child process running this script with --workload cfg3, i.e. exactly as a
        # stand-alone run measures it: in a fresh address space (pools allocated after another
        # workload's were freed measured about 2 % slower).
        del r
        torch.cuda.empty_cache()
        cmd = [sys.executable, os.path.abspath(__file__), "--workload", "cfg3", "--steps",
               str(max(10, min(args.steps, 50))), "--warmup", str(min(args.warmup, 5))]
        if args.no_cpu_baseline:
            cmd.append("--no-cpu-baseline")
        child = subprocess.run(cmd, capture_output=True, text=True)
        lines = [ln for ln in child.stdout.splitlines() if ln.startswith("{")]
        if not lines:
            print("bench.py: the cfg3 run failed:\n" + child.stderr[-2000:], file=sys.stderr)
            sys.exit(1)
        r3 = json.loads(lines[-1])
        res["cfg3"] = {"workload": r3["config"]["workload"], "partition_size": r3["config"]["partition_size"],
                       "num_seqs": r3["config"]["num_seqs"],
                       "total_context_tokens": r3["config"]["total_context_tokens"],
                       "steps": r3["steps"], "attn": r3["attn"], "migration": r3["migration"],
                       "step": r3["step"], "roofline": r3["roofline"],
                       "cpu_baseline": r3["cpu_baseline"], "parity": r3.get("parity"),
                       "box_stream_read": r3.get("box_stream_read")}
        ok = ok and child.returncode == 0 and (r3.get("parity") or {}).get("within_bar", True)
    print(json.dumps(res), flush=True)
    if not ok:
        print("bench.py: attention output outside the parity bar (max-abs 1e-2, rel-L2 5e-3)",
              file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
