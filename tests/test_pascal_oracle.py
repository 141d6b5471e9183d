"""Pins of the scheduler oracle (CPU only): the two instance-selection algorithms on
worked tables, the adaptive-migration example, closed forms for the QoE measure, and
invariants of the queue dynamics on seeded traces."""
import itertools

import numpy as np
import pytest

from oracle import pascal_oracle as po
from paper_2602_11530_amd import workloads as wl

from serving_driver import replay


# ---- Algorithm 1 (instance selection for reasoning requests) ---------------------

def test_alg1_worked_tables():
    f = po.select_reasoning_instance
    # smallest KV footprint among the instances that meet their answering SLO
    assert f([True, True, True], [7, 3, 5]) == 1
    assert f([True, False, True], [7, 3, 5]) == 2      # instance 1 is excluded although it is the emptiest
    assert f([False, False, True], [1, 2, 900]) == 2   # a single candidate wins whatever its footprint
    # nobody meets the SLO: fall back to all instances
    assert f([False, False, False], [7, 3, 5]) == 1
    assert f([True] * 4, [4, 2, 2, 9]) == 1            # tie: lowest index


def test_alg1_against_exhaustive_definition():
    rng = np.random.default_rng(1)
    for _ in range(300):
        n = int(rng.integers(1, 9))
        t = rng.random(n) < 0.6
        m = rng.integers(0, 6, size=n)
        cand = [i for i in range(n) if t[i]] or list(range(n))
        got = po.select_reasoning_instance(list(t), list(m))
        assert got in cand and all(m[got] <= m[i] for i in cand)
        assert all(m[i] > m[got] for i in cand if i < got)


# ---- Algorithm 2 (instance selection for answering requests) --------------------

def test_alg2_worked_tables():
    f = po.select_answering_instance
    # fewest reasoning requests among SLO-compliant instances; a_i plays no part there
    assert f([True, True, True], [4, 1, 2], [0, 50, 0]) == 1
    assert f([True, False, True], [4, 1, 2], [0, 0, 0]) == 2
    # nobody compliant: r_i + a_i decides
    assert f([False] * 3, [4, 1, 2], [0, 5, 1]) == 2    # 4, 6, 3
    assert f([False] * 3, [4, 1, 2], [0, 0, 9]) == 1    # 4, 1, 11
    # r alone would pick 1, r + a picks 0
    assert f([False] * 2, [3, 2], [0, 2]) == 0
    # ties: stay where you are, else lowest index
    assert f([True] * 3, [2, 2, 2], [0, 0, 0], current=2) == 2
    assert f([True] * 3, [2, 2, 2], [0, 0, 0], current=None) == 0
    assert f([True, True, False], [2, 2, 0], [0, 0, 0], current=2) == 0   # current is not a candidate


def test_alg2_against_exhaustive_definition():
    rng = np.random.default_rng(2)
    for _ in range(300):
        n = int(rng.integers(1, 9))
        t = rng.random(n) < 0.5
        r, a = rng.integers(0, 5, size=n), rng.integers(0, 5, size=n)
        cur = int(rng.integers(0, n))
        if t.any():
            cand, key = [i for i in range(n) if t[i]], r
        else:
            cand, key = list(range(n)), r + a
        got = po.select_answering_instance(list(t), list(r), list(a), current=cur)
        assert got in cand and all(key[got] <= key[i] for i in cand)
        if cur in cand and key[cur] == key[got]:
            assert got == cur


# ---- adaptive migration (Section IV-B, the example of its figure) -------------------

def test_adaptive_migration_example():
    """Instance 2 holds the answering requests and its memory is full; instance 0, where
    the request finished reasoning, still has two free slots: Algorithm 2 says 2, the
    override keeps the request on 0."""
    t, r, a = [True] * 3, [2, 1, 0], [0, 0, 3]
    sel = po.select_answering_instance(t, r, a, current=0)
    assert sel == 2
    assert po.adaptive_migration(0, sel, free_current=2, free_selected=0, request_blocks=1, headroom=1) == 0
    # with room at the destination the migration goes ahead
    assert po.adaptive_migration(0, sel, free_current=2, free_selected=4, request_blocks=1, headroom=1) == 2
    # neither has room: Algorithm 2's choice stands
    assert po.adaptive_migration(0, sel, free_current=0, free_selected=0, request_blocks=1, headroom=1) == 2
    assert po.adaptive_migration(1, 1, 0, 0, 5, 1) == 1


def _golden(name):
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)
    return [ln.split("#")[0].split() for ln in open(path) if ln.split("#")[0].strip()]


def test_adaptive_migration_golden_example():
    rows = _golden("adaptive_migration_example.txt")
    inst, (cur, want_alg2, want_final) = rows[:-1], map(int, rows[-1])
    r = [int(x[1]) for x in inst]
    free = [int(x[2]) for x in inst]
    t = [bool(int(x[3])) for x in inst]
    sel = po.select_answering_instance(t, r, [0] * len(r), current=cur)
    assert sel == want_alg2
    # the request occupies at least one slot; any headroom from one slot up gives the same answer
    for headroom in (1, 2):
        assert po.adaptive_migration(cur, sel, free[cur], free[sel], 1, headroom) == want_final


def test_defaults_are_the_papers_constants():
    import inspect
    from paper_2602_11530_amd import sched_binding as sb
    c = {k: float(v) for k, v in _golden("paper_constants.txt")}
    cfg = po.Config()
    assert (cfg.quantum, cfg.demote_tokens, cfg.num_instances, cfg.tpot) == \
        (c["quantum_tokens"], c["demote_tokens"], c["num_instances"], c["target_tpot_s"])
    d = {k: v.default for k, v in inspect.signature(sb.Scheduler.__init__).parameters.items()}
    assert (d["quantum"], d["demote_tokens"], d["num_instances"], d["tpot"]) == \
        (c["quantum_tokens"], c["demote_tokens"], c["num_instances"], c["target_tpot_s"])
    t = inspect.signature(wl.serving_trace).parameters
    assert (t["n_requests"].default, t["prompt"].default, t["lo"].default, t["hi"].default) == \
        (c["trace_requests"], c["prompt_tokens"], c["phase_tokens_min"], c["phase_tokens_max"])
    assert c["qoe_slo"] == 0.95


# ---- QoE and the pacer -----------------------------------------------------------------

def test_qoe_closed_forms():
    tp = 0.1
    on_pace = [2.0 + k * tp for k in range(50)]
    assert po.qoe(on_pace, tp) == pytest.approx(1.0, abs=1e-12)
    # faster than the reader: the pacer buffers, the reader is never starved
    burst = [2.0 + k * 0.01 for k in range(50)]
    assert po.qoe(burst, tp) == pytest.approx(1.0, abs=1e-12)
    assert po.digest_times(burst, tp) == pytest.approx(on_pace)
    # two tokens, the second three periods late: digested area 3, expected area 3 + 2
    assert po.qoe([0.0, 3.0], 1.0) == pytest.approx(0.6)
    # a pause of `gap` after token j delays every later token by gap - (buffer drained)
    N, j, gap = 20, 7, 2.5
    g = [k * 1.0 for k in range(j + 1)] + [j + gap + (k - j - 1) * 1.0 for k in range(j + 1, N)]
    d = po.digest_times(g, 1.0)
    late = gap - 1.0
    assert d[: j + 1] == pytest.approx(list(range(j + 1)))
    assert d[j + 1:] == pytest.approx([k + late for k in range(j + 1, N)])
    T = N - 1 + late
    want = sum(T - x for x in d) / sum(T - k for k in range(N))
    assert po.qoe(g, 1.0) == pytest.approx(want) and want < 1
    # bounds and monotonicity: more delay never raises the score
    rng = np.random.default_rng(3)
    for _ in range(100):
        gaps = rng.exponential(0.1, size=30)
        g = list(np.cumsum(gaps))
        s = po.qoe(g, tp)
        assert 0 < s <= 1 + 1e-12
        g2 = g[:10] + [x + 0.7 for x in g[10:]]
        assert po.qoe(g2, tp) <= s + 1e-12
    assert po.qoe([], tp) == 1.0 and po.qoe([5.0], tp) == 1.0


def test_pacer_release_schedule():
    # a burst of 10 tokens within 0.1 s, pace 1 s: one token becomes visible per second
    g = [5.0 + 0.01 * k for k in range(10)]
    assert [po.visible_tokens(g, 1.0, 5.0 + x) for x in (-0.1, 0.0, 0.99, 1.0, 3.5, 9.0, 100.0)] == \
        [0, 1, 1, 2, 4, 10, 10]
    # slower than the pace: every token is visible the moment it exists
    g = [0.0, 2.0, 4.0]
    assert [po.visible_tokens(g, 1.0, t) for t in (0.0, 1.9, 2.0, 4.0)] == [1, 1, 2, 3]
    # a pause after a burst: the buffer bridges it (4 tokens at once, then nothing for 3.5 s)
    g = [0.0, 0.0, 0.0, 0.0, 3.5]
    assert [po.visible_tokens(g, 1.0, t) for t in (0.0, 1.0, 2.0, 3.0, 3.4, 3.5, 4.0)] == [1, 2, 3, 4, 4, 4, 5]
    assert po.visible_tokens([], 1.0, 9.0) == 0


def test_pacer_lagging():
    # first token at 10.0, pace 0.1: by 10.35 the reader expects tokens 0..3
    assert not po.pacer_lagging(4, 10.0, 10.35, 0.1)
    assert po.pacer_lagging(3, 10.0, 10.35, 0.1)
    assert not po.pacer_lagging(0, 0.0, 99.0, 0.1)     # no answering token yet: no pace to hold
    assert not po.pacer_lagging(1, 10.0, 10.0, 0.1)


# ---- queue dynamics: invariants on seeded traces ----------------------------------------

class Checked(po.Cluster):
    """The oracle with every invariant asserted after each call."""

    def check(self, i):
        cfg, ins = self.cfg, self.inst[i]
        held = [b for rid in list(ins.high) + list(ins.low) for b in self.req[rid].blocks]
        assert len(held) == len(set(held)), "a block belongs to two requests"
        assert sorted(held + ins.free) == list(range(cfg.gpu_blocks)), "blocks leaked or invented"
        for rid in ins.high:
            q = self.req[rid]
            assert q.level == po.HIGH and q.phase == po.REASONING and q.instance == i
        for rid in ins.low:
            q = self.req[rid]
            assert q.level == po.LOW and q.instance == i
            assert q.phase == po.ANSWERING or q.kv_tokens > cfg.demote_tokens
        for rid in list(ins.high) + list(ins.low):
            q = self.req[rid]
            if q.state == po.RESIDENT:
                assert len(q.blocks) >= self.blocks_for(q.kv_tokens) and q.offloaded_blocks == 0
            elif q.state == po.OFFLOADED:
                assert not q.blocks and q.offloaded_blocks == self.blocks_for(q.kv_tokens)
            else:
                assert q.state == po.QUEUED and (not q.blocks or rid in ins.selected)

    def plan(self, i):
        before = {rid: self.req[rid].state for rid in list(self.inst[i].high) + list(self.inst[i].low)}
        order = list(self.inst[i].high) + list(self.inst[i].low)
        rids, lens, ops = super().plan(i)
        self.check(i)
        # priority: nobody is evicted in favour of a request behind it in the order
        first_evicted = min((order.index(op[2]) for op in ops if op[0] == po.OP_OFFLOAD), default=None)
        if first_evicted is not None:
            gained = [order.index(op[2]) for op in ops
                      if op[0] in (po.OP_PREFILL, po.OP_RELOAD, po.OP_GROW)]
            assert gained and min(gained) < first_evicted
            # and everything ahead of the first victim that was resident stayed resident
            for rid in order[:first_evicted]:
                if before[rid] == po.RESIDENT:
                    assert self.req[rid].state == po.RESIDENT
        # each run of evictions serves the request whose op follows it: never one of lower priority
        victims = []
        for op in ops:
            if op[0] == po.OP_OFFLOAD:
                victims.append(op[2])
            elif victims:
                for v in victims:
                    assert self.req[op[2]].level <= self.req[v].level, "evicted for a lower-priority request"
                    assert order.index(op[2]) < order.index(v)
                victims = []
        assert not victims, "an eviction served nobody"
        assert len(set(rids)) == len(rids)
        for rid, L in zip(rids, lens):
            q = self.req[rid]
            assert len(q.blocks) == self.blocks_for(L)
        return rids, lens, ops

    def commit(self, i, now, kinds):
        ops = super().commit(i, now, kinds)
        for j in range(self.cfg.num_instances):
            self.check(j)
        return ops


@pytest.mark.parametrize("gpu_blocks,rate", [(4000, 4.0), (700, 6.0), (300, 3.0)])
def test_queue_dynamics_invariants(gpu_blocks, rate):
    """Ample memory, pressure, and severe pressure (one long request nearly fills an instance)."""
    trace = wl.serving_trace(n_requests=40, rate_per_s=rate, seed=wl.BASE_SEED + 60)
    cfg = po.Config(num_instances=3, gpu_blocks=gpu_blocks, quantum=500, demote_tokens=3000)
    c = Checked(cfg)
    log = replay(c, trace, cfg.num_instances)
    n_off = sum(1 for e in log if e[0] == "plan" for op in e[4] if op[0] == po.OP_OFFLOAD)
    n_rel = sum(1 for e in log if e[0] == "plan" for op in e[4] if op[0] == po.OP_RELOAD)
    n_mig = sum(1 for e in log if e[0] == "commit" for op in e[4] if op[0] in (po.OP_MIGRATE, po.OP_MIGRATE_HOST))
    print(f"blocks={gpu_blocks}: offloads {n_off}, reloads {n_rel}, migrations {n_mig}")
    if gpu_blocks == 4000:
        assert n_off == 0
    else:
        assert n_off > 0 and n_rel > 0
    for rid, q in enumerate(c.req):
        assert q.state == po.FINISHED and not q.blocks
        assert q.reasoning_tokens == trace.reasoning[rid]
        assert len(q.answer_times) == trace.answering[rid]
        assert q.kv_tokens == trace.prompt[rid] + trace.reasoning[rid] + trace.answering[rid] - 1
        assert c.ttft(rid) > 0 and 0 < c.qoe(rid) <= 1 + 1e-12
    for ins in c.inst:
        assert not ins.high and not ins.low and len(ins.free) == gpu_blocks
    # every offload is answered by exactly one reload or host-side hand-over of the same request
    assert n_off == n_rel - sum(1 for e in log if e[0] == "commit" for op in e[4] if op[0] == po.OP_MIGRATE_HOST)


def test_reasoning_is_never_evicted_for_answering():
    """One instance under pressure: reasoning requests take turns among themselves, an
    answering request is pushed out when they need its memory, never the reverse."""
    cfg = po.Config(num_instances=1, gpu_blocks=48, quantum=50, demote_tokens=10**9)
    c = Checked(cfg)
    a, _ = c.submit(160, 0.0)     # 10 blocks each, growing
    b, _ = c.submit(160, 0.0)
    now, evicted_levels = 0.0, []
    for step in range(260):
        rids, lens, ops = c.plan(0)
        evicted_levels += [(c.req[op[2]].level, c.req[op[2]].phase) for op in ops if op[0] == po.OP_OFFLOAD]
        now += 0.03
        kinds = [po.END_OF_REASONING if (r == a and step == 20) else po.TOKEN for r in rids]
        c.commit(0, now, kinds)
        if step == 25:
            c.submit(200, now)    # a newcomer: high priority, may push the answering request out
    assert c.req[a].phase == po.ANSWERING and c.req[b].phase == po.REASONING
    assert c.req[a].preemptions > 0, "the scenario should put the answering request under pressure"
    assert (po.LOW, po.ANSWERING) in evicted_levels


@pytest.mark.parametrize("seed", range(25))
def test_invariants_on_random_walks(seed):
    """The same invariants under arbitrary interleavings and randomly drawn token kinds."""
    rng = np.random.default_rng(2000 + seed)
    n_inst = int(rng.integers(1, 4))
    cfg = po.Config(num_instances=n_inst, gpu_blocks=int(rng.integers(6, 30)),
                    block_tokens=int(rng.choice([1, 4, 16])), quantum=int(rng.integers(1, 10)),
                    demote_tokens=int(rng.integers(8, 120)), headroom_blocks=int(rng.integers(0, 3)),
                    tpot=0.05, max_batch=int(rng.choice([0, 2])))
    c = Checked(cfg)
    cap = cfg.gpu_blocks * cfg.block_tokens
    now, live = 0.0, 0
    for _ in range(300):
        now += float(rng.exponential(0.03))
        if live < 10 and rng.random() < 0.3:
            c.submit(int(rng.integers(1, max(2, cap // 3))), now)
            live += 1
        i = int(rng.integers(0, n_inst))
        rids, lens, _ = c.plan(i)
        kinds = []
        for rid, L in zip(rids, lens):
            u = rng.random()
            if L + 1 >= cap or u < 0.03:
                kinds.append(po.END_OF_SEQUENCE)
                live -= 1
            elif c.req[rid].phase == po.REASONING and u < 0.10:
                kinds.append(po.END_OF_REASONING)
            else:
                kinds.append(po.TOKEN)
        c.commit(i, now, kinds)


# ---- queue dynamics: hand-worked tables -------------------------------------------------
# Every expected value below was worked out on paper from the paper's words: a request that
# has consumed all of its token quantum loses priority inside its queue and requests take
# their quanta in circular order (Sections II-B, V-A); under memory pressure the
# lowest-priority request is the one evicted (Section II-B); a reasoning request is demoted
# when its KV cache exceeds the threshold (Section IV-C); a_i counts the answering requests
# that have not yet exhausted their first quantum (Section IV-B).  Nothing here is computed
# by the code under test.

P, O, G_, F = po.OP_PREFILL, po.OP_OFFLOAD, po.OP_GROW, po.OP_FREE


def _one_instance(**kw):
    base = dict(num_instances=1, gpu_blocks=64, block_tokens=16, quantum=3, demote_tokens=10 ** 9)
    base.update(kw)
    return po.Cluster(po.Config(**base))


def test_table_quantum_of_three_two_requests():
    """Quantum 3.  Request 0 arrives one iteration before request 1.  The third token of a
    quantum exhausts it (not the fourth): the request goes to the back right then."""
    c = _one_instance()
    c.submit(16, 0.0)
    want_batch = [[0], [0, 1], [0, 1], [1, 0], [0, 1], [0, 1], [1, 0]]
    want_lens = [[16], [17, 16], [18, 17], [18, 19], [20, 19], [21, 20], [21, 22]]
    want_queue = [[0], [0, 1], [1, 0], [0, 1], [0, 1], [1, 0], [0, 1]]
    want_quanta = [(0, 0), (0, 0), (1, 0), (1, 1), (1, 1), (2, 1), (2, 2)]   # completed quanta of 0, 1
    for it in range(7):
        rids, lens, _ = c.plan(0)
        assert (rids, lens) == (want_batch[it], want_lens[it]), f"iteration {it + 1}"
        c.commit(0, 0.1 * (it + 1), [po.TOKEN] * len(rids))
        assert list(c.inst[0].high) == want_queue[it], f"queue after iteration {it + 1}"
        assert (c.req[0].quanta_done, c.req[1].quanta_done if len(c.req) > 1 else 0) == want_quanta[it]
        if it == 0:
            c.submit(16, 0.1)                       # request 1 arrives after the first iteration


def test_table_circular_order_under_a_batch_cap():
    """One request per iteration, quantum 3: three tokens each, in turn."""
    c = _one_instance(max_batch=1)
    c.submit(16, 0.0)
    c.submit(16, 0.0)
    ran = []
    for it in range(12):
        rids, _, _ = c.plan(0)
        ran += rids
        c.commit(0, 0.1 * (it + 1), [po.TOKEN] * len(rids))
    assert ran == [0, 0, 0, 1, 1, 1, 0, 0, 0, 1, 1, 1]


def test_table_demotion_needs_more_than_the_threshold():
    """Threshold 20 tokens, prompt 18: still high-priority with exactly 20 tokens of KV cache,
    demoted by the token that makes it 21, in that very iteration."""
    c = _one_instance(quantum=500, demote_tokens=20)
    c.submit(18, 0.0)
    levels, kv = [], []
    for it in range(5):
        rids, lens, _ = c.plan(0)
        assert rids == [0]
        c.commit(0, 0.1 * (it + 1), [po.TOKEN])
        levels.append(c.req[0].level)
        kv.append(c.req[0].kv_tokens)
    assert kv == [18, 19, 20, 21, 22]
    assert levels == [po.HIGH, po.HIGH, po.HIGH, po.LOW, po.LOW]
    assert list(c.inst[0].high) == [] and list(c.inst[0].low) == [0]
    assert c.req[0].phase == po.REASONING          # still reasoning, only treated as low priority
    assert c.r(0) == 0                              # and no longer counted among the reasoning requests


def test_table_victim_is_the_last_in_order():
    """Three requests of one block each fill a three-block instance.  When the first needs a
    second block, the request at the END of the round-robin order is evicted (request 2), not the
    one right behind it (request 1); request 1 then finds no block either and waits, resident."""
    c = _one_instance(gpu_blocks=3, quantum=500)
    for _ in range(3):
        c.submit(16, 0.0)
    rids, lens, ops = c.plan(0)
    assert (rids, lens) == ([0, 1, 2], [16, 16, 16])
    assert ops == [(P, 0, 0, (0,), -1, ()), (P, 0, 1, (1,), -1, ()), (P, 0, 2, (2,), -1, ())]
    c.commit(0, 0.1, [po.TOKEN] * 3)
    rids, lens, ops = c.plan(0)
    assert (rids, lens) == ([0], [17])
    assert ops == [(O, 0, 2, (2,), -1, ()), (G_, 0, 0, (2,), -1, ())]
    assert [c.req[r].state for r in range(3)] == [po.RESIDENT, po.RESIDENT, po.OFFLOADED]
    assert (c.req[2].preemptions, c.req[2].offloaded_blocks, c.req[1].preemptions) == (1, 1, 0)
    c.commit(0, 0.2, [po.TOKEN])
    rids, lens, ops = c.plan(0)                    # nothing changes hands: 1 and 2 keep waiting
    assert (rids, lens, ops) == ([0], [18], [])
    c.commit(0, 0.3, [po.TOKEN])


def test_table_victim_follows_round_robin_order_not_arrival():
    """Quantum 2.  Request 0 arrives first and uses up its quantum, which puts it behind 1 and
    2; when memory runs out it is request 0 that goes, although it is the oldest."""
    c = _one_instance(gpu_blocks=4, quantum=2)
    c.submit(16, 0.0)
    assert c.plan(0) == ([0], [16], [(P, 0, 0, (0,), -1, ())])
    c.commit(0, 0.1, [po.TOKEN])
    c.submit(16, 0.1)
    c.submit(16, 0.1)
    rids, lens, ops = c.plan(0)
    assert (rids, lens) == ([0, 1, 2], [17, 16, 16])
    assert ops == [(G_, 0, 0, (1,), -1, ()), (P, 0, 1, (2,), -1, ()), (P, 0, 2, (3,), -1, ())]
    c.commit(0, 0.2, [po.TOKEN] * 3)
    assert list(c.inst[0].high) == [1, 2, 0]       # 0 has had its two tokens
    rids, lens, ops = c.plan(0)
    assert (rids, lens) == ([1, 2], [17, 17])
    assert [(op[0], op[2]) for op in ops] == [(O, 0), (G_, 1), (G_, 2)]
    assert ops[0][3] == (0, 1)                      # both of request 0's blocks are given up
    assert sorted(ops[1][3] + ops[2][3]) == [0, 1]  # and handed to 1 and 2
    assert c.req[0].state == po.OFFLOADED


def test_table_fresh_answering_requests():
    """a_i: answering requests that have not used up their first quantum (3 tokens here)."""
    c = _one_instance()
    c.submit(16, 0.0)
    now = 0.0

    def step(kinds):
        nonlocal now
        rids, _, _ = c.plan(0)
        now += 0.1
        c.commit(0, now, [kinds.get(r, po.TOKEN) for r in rids])
        return rids

    step({})                                        # prefill: first reasoning token
    assert (c.r(0), c.a(0)) == (1, 0)
    step({0: po.END_OF_REASONING})                  # the closing token of the reasoning phase
    assert (c.r(0), c.a(0)) == (0, 1) and list(c.inst[0].low) == [0]
    step({}); assert c.a(0) == 1                    # 1st answering token
    step({}); assert c.a(0) == 1                    # 2nd
    step({}); assert c.a(0) == 0                    # 3rd: first quantum exhausted
    assert len(c.req[0].answer_times) == 3
    c.submit(16, now)                               # a newcomer reasons for two iterations ...
    assert (c.r(0), c.a(0)) == (1, 0)
    assert step({}) == [1, 0]                       # reasoning runs ahead of answering
    step({1: po.END_OF_REASONING})
    assert (c.r(0), c.a(0)) == (0, 1)               # ... and is the only fresh answering request
    assert list(c.inst[0].low) == [0, 1]
    step({}); step({}); assert c.a(0) == 1
    step({}); assert c.a(0) == 0
