"""Plain-Python checker for the phase-aware scheduler that drives the KV kernels.

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` alone, never by the product
package, and it shares no code with the C++ scheduler library.

What follows the paper directly (Section IV), in its notation:

* ``select_reasoning_instance(t, m)`` — Algorithm 1: E = {i : t_i}; E = I when
  that is empty; argmin over E of m_i (KV memory on GPU + CPU).
* ``select_answering_instance(t, r, a)`` — Algorithm 2: E = {i : t_i}; when
  that is empty E = I and r_i <- r_i + a_i; argmin over E of r_i.
* ``adaptive_migration`` — Section IV-B: at the phase transition the request
  stays where it is when its current instance has sufficient GPU memory and
  the selected one has not.
* Two queues per instance, reasoning requests in the high-priority one, answering
  requests in the low-priority one, round-robin inside each with a token
  quantum (500 in Section V-A); a reasoning request whose KV cache exceeds a
  threshold (5000 tokens) is demoted to the low-priority queue (Section IV-C).
* ``qoe`` — Section II-C (its QoE figure): area under the user-digested token curve over
  the area under the user-expected curve, computed from TPOT only and starting
  at the first answering token (Section V-A, "Metric").
* t_i — Section IV-B: an instance violates its answering SLO when its token
  pacer holds too few tokens, i.e. generation is behind the user's pace.

Where the paper is silent this file takes a reading of its own; each is marked
"reading" where it is applied.  Pins (tests/test_pascal_oracle.py):
worked tables for both algorithms, the adaptive-migration example of the figure in Section IV-B,
closed forms for QoE, hand-worked tables for the queue dynamics (a quantum of three
tokens over seven iterations, circular order under a batch cap, demotion only
above the threshold, the eviction victim is the last request in round-robin
order, a_i counts first-quantum answering requests only), and invariants on
seeded traces and random walks (capacity never exceeded, block ids unique,
priority respected, every token accounted for).  What stays a reading rather
than a pinned value: tie-breaks, what counts towards m_i, the allocator's id
order.
"""
from __future__ import annotations

import math
from collections import deque
from dataclasses import dataclass, field
from typing import Deque, Dict, List, Optional, Sequence, Tuple

# ---------------------------------------------------------------- Algorithms 1, 2


def select_reasoning_instance(t: Sequence[bool], m: Sequence[int]) -> int:
    """Algorithm 1.  reading: ties go to the lowest instance index."""
    I = range(len(t))
    E = [i for i in I if t[i]]
    if not E:
        E = list(I)
    best = E[0]
    for i in E:
        if m[i] < m[best]:
            best = i
    return best


def select_answering_instance(t: Sequence[bool], r: Sequence[int], a: Sequence[int],
                              current: Optional[int] = None) -> int:
    """Algorithm 2.  reading: among equal minima the request's current instance
    wins (no transfer for nothing), then the lowest index."""
    I = range(len(t))
    r = list(r)
    E = [i for i in I if t[i]]
    if not E:
        E = list(I)
        for i in E:
            r[i] = r[i] + a[i]
    lowest = min(r[i] for i in E)
    if current is not None and current in E and r[current] == lowest:
        return current
    return next(i for i in E if r[i] == lowest)


def adaptive_migration(current: int, selected: int, free_current: int, free_selected: int,
                       request_blocks: int, headroom: int) -> int:
    """Section IV-B, adaptive migration.  reading: "sufficient GPU memory" means, on
    the current instance (which already holds the request), at least `headroom`
    free blocks; on the selected one, room for the request's blocks plus
    `headroom`."""
    if selected == current:
        return current
    current_ok = free_current >= headroom
    selected_ok = free_selected >= request_blocks + headroom
    if current_ok and not selected_ok:
        return current
    return selected


# ---------------------------------------------------------------- token pacer, QoE


def digest_times(g: Sequence[float], tpot: float) -> List[float]:
    """When the user reads each answering token: no faster than one per `tpot`
    and never before it exists (the pacer buffers early tokens, Section II-C)."""
    d: List[float] = []
    for k, gk in enumerate(g):
        d.append(gk if k == 0 else max(gk, d[-1] + tpot))
    return d


def qoe(g: Sequence[float], tpot: float) -> float:
    """Area under the digested-token step curve over the area under the expected
    one, both from the first answering token to the moment the user has read the
    last one.  reading: step curves; token k (from 0) is expected at g[0] + k*tpot."""
    if len(g) <= 1:
        return 1.0
    d = digest_times(g, tpot)
    T = d[-1]
    digested = sum(T - dk for dk in d)
    expected = sum(T - (g[0] + k * tpot) for k in range(len(g)))
    return digested / expected if expected > 0 else 1.0


def visible_tokens(g: Sequence[float], tpot: float, now: float) -> int:
    """Tokens the pacer has released by `now`: those whose reading time has come."""
    return sum(1 for dk in digest_times(g, tpot) if dk <= now)


def pacer_lagging(n_answer_tokens: int, t_first: float, now: float, tpot: float) -> bool:
    """The pacer has run dry: by `now` the user expects more tokens than exist."""
    if n_answer_tokens < 1:
        return False
    expected = 1 + math.floor((now - t_first) / tpot)
    return n_answer_tokens < expected


# ---------------------------------------------------------------- queue dynamics

REASONING, ANSWERING = 0, 1
HIGH, LOW = 0, 1
QUEUED, RESIDENT, OFFLOADED, FINISHED = 0, 1, 2, 3
TOKEN, END_OF_REASONING, END_OF_SEQUENCE = 0, 1, 2
OP_OFFLOAD, OP_RELOAD, OP_PREFILL, OP_GROW, OP_MIGRATE, OP_MIGRATE_HOST, OP_FREE = 1, 2, 3, 4, 5, 6, 7


@dataclass
class Config:
    num_instances: int = 8
    gpu_blocks: int = 1024          # KV blocks per instance
    block_tokens: int = 16
    quantum: int = 500              # tokens, both queues (Section V-A)
    demote_tokens: int = 5000       # Section V-A
    headroom_blocks: int = 1
    tpot: float = 0.1               # target seconds per answering token (100 ms, Section III)
    max_batch: int = 0              # 0 = no cap
    migration: bool = True          # False: the "no migration" ablation of Section V-D
    adaptive: bool = True           # False: Algorithm 2's choice without the adaptive override


@dataclass
class Request:
    rid: int
    arrival: float
    prompt: int
    instance: int
    phase: int = REASONING
    level: int = HIGH
    state: int = QUEUED
    kv_tokens: int = 0
    blocks: List[int] = field(default_factory=list)
    offloaded_blocks: int = 0
    quantum_used: int = 0
    quanta_done: int = 0
    reasoning_tokens: int = 0
    answer_times: List[float] = field(default_factory=list)
    preemptions: int = 0
    migrations: int = 0
    finish: float = -1.0


@dataclass
class Instance:
    free: List[int]                 # stack: the last entry is handed out next
    high: Deque[int] = field(default_factory=deque)
    low: Deque[int] = field(default_factory=deque)
    selected: List[int] = field(default_factory=list)


Op = Tuple[int, int, int, Tuple[int, ...], int, Tuple[int, ...]]
# (kind, instance, request, blocks, other instance or -1, blocks there)


class Cluster:
    def __init__(self, cfg: Config):
        self.cfg = cfg
        # reading: blocks are handed out lowest id first; freed blocks are reused last-freed first
        self.inst = [Instance(free=list(range(cfg.gpu_blocks - 1, -1, -1)))
                     for _ in range(cfg.num_instances)]
        self.req: List[Request] = []

    # -- per-instance signals of Section IV-B ------------------------------------
    def blocks_for(self, tokens: int) -> int:
        return -(-tokens // self.cfg.block_tokens)

    def t(self, i: int, now: float) -> bool:
        for rid in self.inst[i].low:
            q = self.req[rid]
            if q.phase == ANSWERING and q.answer_times and \
                    pacer_lagging(len(q.answer_times), q.answer_times[0], now, self.cfg.tpot):
                return False
        return True

    def m(self, i: int) -> int:
        """KV memory of the instance in blocks, GPU + CPU.  reading: the prompt of a
        request that has not started yet counts too (its memory is committed)."""
        total = 0
        for rid in list(self.inst[i].high) + list(self.inst[i].low):
            q = self.req[rid]
            if q.state == QUEUED:
                total += self.blocks_for(q.prompt)
            elif q.state == RESIDENT:
                total += len(q.blocks)
            else:
                total += q.offloaded_blocks
        return total

    def r(self, i: int) -> int:
        return len(self.inst[i].high)

    def a(self, i: int) -> int:
        return sum(1 for rid in self.inst[i].low if self.req[rid].quanta_done == 0)

    def free_blocks(self, i: int) -> int:
        return len(self.inst[i].free)

    # -- arrivals: Algorithm 1 ---------------------------------------------------
    def submit(self, prompt: int, now: float) -> Tuple[int, int]:
        n = self.cfg.num_instances
        i = select_reasoning_instance([self.t(j, now) for j in range(n)],
                                      [self.m(j) for j in range(n)])
        rid = len(self.req)
        self.req.append(Request(rid, now, prompt, i))
        self.inst[i].high.append(rid)
        return rid, i

    # -- one iteration of an instance: who runs, who is evicted -----------------
    def plan(self, i: int) -> Tuple[List[int], List[int], List[Op]]:
        """Returns (requests of this iteration's batch, their context lengths after the
        iteration, data-movement ops in execution order).

        reading: requests are considered in priority order (high-priority queue, then
        low-priority queue, each in round-robin order).  Each needs the blocks that
        hold its KV cache after this iteration; when they are not free, resident
        requests of lower priority are evicted, the last in order first, and never
        a request of higher priority.  Nobody is evicted for a request that would
        not fit even then: it waits."""
        ins, cfg = self.inst[i], self.cfg
        assert not ins.selected, "commit() must follow plan()"
        order = list(ins.high) + list(ins.low)
        ops: List[Op] = []
        selected: List[int] = []
        evicted = set()
        for pos, rid in enumerate(order):
            q = self.req[rid]
            if rid in evicted:
                continue                                  # not twice in one iteration
            after = q.prompt if q.state == QUEUED else q.kv_tokens + 1
            extra = self.blocks_for(after) - len(q.blocks)
            reclaimable = len(ins.free) + sum(len(self.req[v].blocks) for v in order[pos + 1:]
                                              if self.req[v].state == RESIDENT)
            if extra > reclaimable:
                continue                                  # blocked this iteration
            back = len(order) - 1
            while extra > len(ins.free) and back > pos:
                v = self.req[order[back]]
                back -= 1
                if v.state != RESIDENT:
                    continue
                ops.append((OP_OFFLOAD, i, v.rid, tuple(v.blocks), -1, ()))
                ins.free.extend(v.blocks)
                v.offloaded_blocks = len(v.blocks)
                v.blocks = []
                v.state = OFFLOADED
                v.preemptions += 1
                evicted.add(v.rid)
            got = [ins.free.pop() for _ in range(extra)]
            if q.state == QUEUED:
                ops.append((OP_PREFILL, i, rid, tuple(got), -1, ()))
            elif q.state == OFFLOADED:
                n_old = q.offloaded_blocks
                ops.append((OP_RELOAD, i, rid, tuple(got[:n_old]), -1, ()))
                if extra > n_old:
                    ops.append((OP_GROW, i, rid, tuple(got[n_old:]), -1, ()))
                q.offloaded_blocks = 0
                q.state = RESIDENT
            elif extra:
                ops.append((OP_GROW, i, rid, tuple(got), -1, ()))
            q.blocks.extend(got)
            selected.append(rid)
            if cfg.max_batch and len(selected) == cfg.max_batch:
                break
        ins.selected = selected
        lens = [self.req[r].prompt if self.req[r].state == QUEUED else self.req[r].kv_tokens + 1
                for r in selected]
        return selected, lens, ops

    # -- the iteration's tokens come back ----------------------------------------
    def commit(self, i: int, now: float, kinds: Sequence[int]) -> List[Op]:
        ins, cfg = self.inst[i], self.cfg
        assert len(kinds) == len(ins.selected)
        ops: List[Op] = []
        for rid, kind in zip(ins.selected, kinds):
            q = self.req[rid]
            if q.state == QUEUED:
                q.state, q.kv_tokens = RESIDENT, q.prompt
            else:
                q.kv_tokens += 1
            if q.phase == REASONING:
                q.reasoning_tokens += 1
            else:
                q.answer_times.append(now)
            queue = ins.high if q.level == HIGH else ins.low
            q.quantum_used += 1
            if q.quantum_used >= cfg.quantum:             # quantum exhausted: to the back
                q.quantum_used = 0
                q.quanta_done += 1
                queue.remove(rid)
                queue.append(rid)
            if kind == END_OF_SEQUENCE:
                queue.remove(rid)
                ops.append((OP_FREE, i, rid, tuple(q.blocks), -1, ()))
                ins.free.extend(q.blocks)
                q.blocks, q.state, q.finish = [], FINISHED, now
            elif kind == END_OF_REASONING and q.phase == REASONING:
                queue.remove(rid)
                ops.extend(self._phase_transition(q, now))
            elif q.phase == REASONING and q.level == HIGH and q.kv_tokens > cfg.demote_tokens:
                ins.high.remove(rid)                      # Section IV-C: conditional demotion
                ins.low.append(rid)
                q.level, q.quantum_used, q.quanta_done = LOW, 0, 0
        ins.selected = []
        return ops

    def _phase_transition(self, q: Request, now: float) -> List[Op]:
        """Algorithm 2, then the adaptive override; the request has already left its queue."""
        n, cur = self.cfg.num_instances, q.instance
        sel = cur
        if self.cfg.migration:
            sel = select_answering_instance([self.t(j, now) for j in range(n)],
                                            [self.r(j) for j in range(n)],
                                            [self.a(j) for j in range(n)], current=cur)
        dst = sel
        if self.cfg.adaptive:
            dst = adaptive_migration(cur, sel, self.free_blocks(cur), self.free_blocks(sel),
                                     len(q.blocks), self.cfg.headroom_blocks)
        q.phase, q.level, q.quantum_used, q.quanta_done = ANSWERING, LOW, 0, 0
        ops: List[Op] = []
        if dst != cur:
            src_blocks = tuple(q.blocks)
            self.inst[cur].free.extend(q.blocks)
            d = self.inst[dst]
            if len(d.free) >= len(src_blocks):
                got = tuple(d.free.pop() for _ in src_blocks)
                ops.append((OP_MIGRATE, cur, q.rid, src_blocks, dst, got))
                q.blocks = list(got)
            else:                                         # arrives in the destination's host store
                ops.append((OP_MIGRATE_HOST, cur, q.rid, src_blocks, dst, ()))
                q.offloaded_blocks, q.blocks, q.state = len(src_blocks), [], OFFLOADED
            q.instance = dst
            q.migrations += 1
        self.inst[dst].low.append(q.rid)
        return ops

    # -- per-request results -----------------------------------------------------
    def ttft(self, rid: int) -> float:
        q = self.req[rid]
        return q.answer_times[0] - q.arrival if q.answer_times else -1.0

    def qoe(self, rid: int) -> float:
        return qoe(self.req[rid].answer_times, self.cfg.tpot)
