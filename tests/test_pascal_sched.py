"""The C++ scheduler library against the Python oracle (CPU only): every decision of a
replayed trace — routing, batches, context lengths, data-movement orders and their block
ids, migrations — must be identical, and the per-request results equal."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import pascal_oracle as po
from paper_2602_11530_amd import sched_binding as sb
from paper_2602_11530_amd import workloads as wl

from serving_driver import replay

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_match_header():
    text = open(os.path.join(ROOT, "include", "pascal_sched.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(pascal_[a-z_]+)\s*\(", text))
    assert declared == set(sb.EXPORTS)
    L = sb.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert ctypes.sizeof(sb.Config) == 40 and ctypes.sizeof(sb.Op) == 32
    assert ctypes.sizeof(sb.RequestInfo) == 80


def test_constants_agree_with_header():
    text = open(os.path.join(ROOT, "include", "pascal_sched.h")).read()
    defs = {k: int(v.strip("()")) for k, v in re.findall(r"#define (PASCAL_[A-Z_]+) (\(?-?\d+\)?)", text)}
    assert (defs["PASCAL_TOKEN"], defs["PASCAL_END_OF_REASONING"], defs["PASCAL_END_OF_SEQUENCE"]) == \
        (sb.TOKEN, sb.END_OF_REASONING, sb.END_OF_SEQUENCE) == (po.TOKEN, po.END_OF_REASONING, po.END_OF_SEQUENCE)
    for name in ("OFFLOAD", "RELOAD", "PREFILL", "GROW", "MIGRATE", "MIGRATE_HOST", "FREE"):
        assert defs["PASCAL_OP_" + name] == getattr(sb, "OP_" + name) == getattr(po, "OP_" + name)


def test_argument_errors():
    L = sb.lib()
    with pytest.raises(sb.SchedError) as e:
        sb.Scheduler(num_instances=0)
    assert e.value.status == -2
    with pytest.raises(sb.SchedError):
        sb.Scheduler(tpot=0.0)
    s = sb.Scheduler(num_instances=2, gpu_blocks=8, block_tokens=16)
    with pytest.raises(sb.SchedError) as e:
        s.submit(0, 0.0)
    assert e.value.status == -2
    with pytest.raises(sb.SchedError) as e:
        s.submit(16 * 8 + 1, 0.0)          # can never fit an instance
    assert e.value.status == -4
    with pytest.raises(sb.SchedError) as e:
        s.commit(0, 0.0, [])               # nothing planned
    assert e.value.status == -3
    rid, inst = s.submit(40, 0.0)
    rids, lens, ops = s.plan(inst)
    assert rids == [rid] and lens == [40] and ops == [(sb.OP_PREFILL, inst, rid, (0, 1, 2), -1, ())]
    with pytest.raises(sb.SchedError) as e:
        s.plan(inst)                       # commit must come first
    assert e.value.status == -3
    with pytest.raises(sb.SchedError) as e:
        s.commit(inst, 0.1, [0, 0])        # one entry per batch member
    assert e.value.status == -2
    with pytest.raises(sb.SchedError) as e:
        s.commit(inst, 0.1, [7])
    assert e.value.status == -2
    with pytest.raises(sb.SchedError) as e:
        s.block_tables(inst, 1, 2)         # the row needs 3 entries
    assert e.value.status == -4
    assert s.block_tables(inst, 1, 4, fill=-7).tolist() == [[0, 1, 2, -7]]
    assert s.commit(inst, 0.1, [0]) == []
    with pytest.raises(sb.SchedError):
        s.plan(5)
    with pytest.raises(sb.SchedError):
        s.request(99)
    assert L.pascal_status_string(-3) != L.pascal_status_string(-99)


class Both:
    """Feeds the library and the oracle the same calls and compares every answer."""

    def __init__(self, **kw):
        self.lib = sb.Scheduler(**kw)
        self.ref = po.Cluster(po.Config(num_instances=kw["num_instances"], gpu_blocks=kw["gpu_blocks"],
                                        block_tokens=kw.get("block_tokens", 16),
                                        quantum=kw.get("quantum", 500),
                                        demote_tokens=kw.get("demote_tokens", 5000),
                                        headroom_blocks=kw.get("headroom_blocks", 1),
                                        tpot=kw.get("tpot", 0.1), max_batch=kw.get("max_batch", 0),
                                        migration=kw.get("migration", True),
                                        adaptive=kw.get("adaptive", True)))
        self.n = kw["num_instances"]
        self.calls = 0

    def submit(self, prompt, now):
        a, b = self.lib.submit(prompt, now), self.ref.submit(prompt, now)
        assert a == b, f"routing differs for request {b[0]}: library {a}, oracle {b}"
        return a

    def plan(self, i):
        a, b = self.lib.plan(i), self.ref.plan(i)
        assert a[0] == b[0] and a[1] == b[1], f"batch differs on instance {i} (call {self.calls})"
        assert a[2] == b[2], f"orders differ on instance {i} (call {self.calls}): {a[2]} vs {b[2]}"
        if a[0] and self.calls % 50 == 0:
            maxb = max(len(self.ref.req[r].blocks) for r in a[0]) + 1
            t = self.lib.block_tables(i, len(a[0]), maxb)
            for row, rid in zip(t, a[0]):
                blocks = self.ref.req[rid].blocks
                assert row[:len(blocks)].tolist() == blocks and (row[len(blocks):] == -1).all()
        self.calls += 1
        return a

    def commit(self, i, now, kinds):
        a, b = self.lib.commit(i, now, kinds), self.ref.commit(i, now, kinds)
        assert a == b, f"commit orders differ on instance {i}: {a} vs {b}"
        if self.calls % 200 == 0:
            for j in range(self.n):
                want = (self.ref.t(j, now), self.ref.m(j), self.ref.r(j), self.ref.a(j), self.ref.free_blocks(j))
                assert self.lib.signals(j, now) == want
        return a


@pytest.mark.parametrize("kw,n_requests,rate", [
    (dict(num_instances=8, gpu_blocks=2000), 120, 12.0),                      # the paper's 8 instances
    (dict(num_instances=3, gpu_blocks=600, demote_tokens=3000), 40, 6.0),     # memory pressure, demotion
    (dict(num_instances=2, gpu_blocks=300, quantum=100, headroom_blocks=8), 30, 2.0),
    (dict(num_instances=4, gpu_blocks=400, max_batch=3, tpot=0.02), 40, 8.0), # capped batch, strict pace
    (dict(num_instances=3, gpu_blocks=600, migration=False), 40, 6.0),        # ablation: no migration
    (dict(num_instances=3, gpu_blocks=600, adaptive=False), 40, 6.0),         # ablation: no adaptive override
])
def test_library_equals_oracle_on_traces(kw, n_requests, rate):
    trace = wl.serving_trace(n_requests=n_requests, rate_per_s=rate, seed=wl.BASE_SEED + 61)
    both = Both(**kw)
    log = replay(both, trace, kw["num_instances"])
    kinds = {}
    for e in log:
        if e[0] in ("plan", "commit"):
            for op in e[4]:
                kinds[op[0]] = kinds.get(op[0], 0) + 1
    print(f"{kw}: {len(log)} calls, orders by kind {dict(sorted(kinds.items()))}")
    assert kinds.get(sb.OP_PREFILL) == n_requests and kinds.get(sb.OP_FREE) == n_requests
    if not kw.get("migration", True):
        assert sb.OP_MIGRATE not in kinds and sb.OP_MIGRATE_HOST not in kinds
    for rid in range(n_requests):
        info, q = both.lib.request(rid), both.ref.req[rid]
        assert info.state == sb.FINISHED == q.state
        assert (info.instance, info.kv_tokens, info.reasoning_tokens, info.answering_tokens,
                info.preemptions, info.migrations) == \
               (q.instance, q.kv_tokens, q.reasoning_tokens, len(q.answer_times), q.preemptions, q.migrations)
        assert info.arrival == q.arrival and info.finish == q.finish
        assert info.ttft == both.ref.ttft(rid)
        assert info.qoe == pytest.approx(both.ref.qoe(rid), rel=1e-12, abs=0)
        assert both.lib.request_blocks(rid) == []


@pytest.mark.parametrize("seed", range(40))
def test_library_equals_oracle_on_random_walks(seed):
    """Arbitrary interleavings of arrivals and iterations, token kinds drawn at random (so
    phase changes and completions hit every queue state), tiny pools, every knob varied."""
    rng = np.random.default_rng(1000 + seed)
    n_inst = int(rng.integers(1, 5))
    kw = dict(num_instances=n_inst, gpu_blocks=int(rng.integers(6, 40)), block_tokens=int(rng.choice([1, 4, 16])),
              quantum=int(rng.integers(1, 12)), demote_tokens=int(rng.integers(8, 200)),
              headroom_blocks=int(rng.integers(0, 4)), tpot=float(rng.choice([0.01, 0.05, 0.3])),
              max_batch=int(rng.choice([0, 0, 1, 3])), migration=bool(rng.random() < 0.8),
              adaptive=bool(rng.random() < 0.8))
    both = Both(**kw)
    cap_tokens = kw["gpu_blocks"] * kw["block_tokens"]
    now, live = 0.0, 0
    for step in range(400):
        now += float(rng.exponential(0.03))
        if live < 12 and rng.random() < 0.25:
            both.submit(int(rng.integers(1, max(2, cap_tokens // 3))), now)
            live += 1
        i = int(rng.integers(0, n_inst))
        rids, lens, _ = both.plan(i)
        kinds = []
        for rid, L in zip(rids, lens):
            q = both.ref.req[rid]
            u = rng.random()
            if L + 1 >= cap_tokens or u < 0.03:         # must stop before it outgrows the pool
                kinds.append(sb.END_OF_SEQUENCE)
                live -= 1
            elif q.phase == po.REASONING and u < 0.10:
                kinds.append(sb.END_OF_REASONING)
            else:
                kinds.append(sb.TOKEN)
        both.commit(i, now, kinds)
        for j in range(n_inst):
            assert both.lib.signals(j, now) == (both.ref.t(j, now), both.ref.m(j), both.ref.r(j),
                                                both.ref.a(j), both.ref.free_blocks(j))
    for rid, q in enumerate(both.ref.req):
        info = both.lib.request(rid)
        assert (info.state, info.phase, info.level, info.instance, info.kv_tokens, info.n_blocks,
                info.preemptions, info.migrations) == \
               (q.state, q.phase, q.level, q.instance, q.kv_tokens, len(q.blocks), q.preemptions, q.migrations)
        assert both.lib.request_blocks(rid) == q.blocks
        assert info.qoe == pytest.approx(both.ref.qoe(rid), rel=1e-12)
        for t in (q.arrival, now / 2, now, now + 50.0):
            assert both.lib.visible_tokens(rid, t) == po.visible_tokens(q.answer_times, kw["tpot"], t)


def test_host_fuzz_under_sanitizers(tmp_path):
    """The scheduler's C++ source compiled with AddressSanitizer and UBSan into a small stress
    program (tests/sched_fuzz.cpp): random arrivals, iterations and token kinds on tiny pools,
    block conservation checked after every call."""
    import subprocess
    exe = str(tmp_path / "sched_fuzz")
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-static-libasan", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "sched_fuzz.cpp"),
                           os.path.join(ROOT, "paper_2602_11530_amd", "csrc", "pascal_sched.cpp"), "-o", exe])
    p = subprocess.run([exe, "20"], capture_output=True, text=True, timeout=300)
    assert p.returncode == 0 and p.stdout.strip() == "clean", p.stderr[-2000:]
