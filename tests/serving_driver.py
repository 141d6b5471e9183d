"""Replays a synthetic trace through a scheduler (the C++ library's binding or the
Python oracle: both expose submit / plan / commit) under a synthetic iteration-time
model, and records everything the scheduler decided.  Test helper only."""
from typing import Callable, List, Optional

TOKEN, END_OF_REASONING, END_OF_SEQUENCE = 0, 1, 2


def iteration_seconds(lens) -> float:
    """Decode iteration time: a fixed part (weights, projections) plus attention time
    proportional to the KV footprint of the batch (memory-bandwidth-bound decode)."""
    return 0.02 + 4.5e-8 * float(sum(lens))


def replay(sched, trace, num_instances: int, on_ops: Optional[Callable] = None,
           on_batch: Optional[Callable] = None, max_iterations: int = 2_000_000) -> List[tuple]:
    """Returns the log: ("submit", rid, inst), ("plan", inst, rids, lens, ops),
    ("commit", inst, now, kinds, ops) in order."""
    log: List[tuple] = []
    n = len(trace)
    produced_r = [0] * n      # reasoning tokens emitted so far, per request
    produced_a = [0] * n
    clock = [0.0] * num_instances
    nxt, done, it = 0, 0, 0
    while done < n:
        it += 1
        assert it <= max_iterations, "the trace does not drain"
        i = min(range(num_instances), key=lambda j: (clock[j], j))
        while nxt < n and trace.arrival[nxt] <= clock[i]:
            rid, inst = sched.submit(int(trace.prompt[nxt]), float(trace.arrival[nxt]))
            assert rid == nxt
            log.append(("submit", rid, inst))
            nxt += 1
        rids, lens, ops = sched.plan(i)
        log.append(("plan", i, tuple(rids), tuple(lens), tuple(ops)))
        if on_ops:
            on_ops(ops)
        if not rids:
            # idle: wake up at the next arrival, or a little later if others are still busy
            clock[i] = max(clock[i] + 0.01, float(trace.arrival[nxt]) if nxt < n else 0.0)
            sched.commit(i, clock[i], [])
            continue
        if on_batch:
            on_batch(i, rids, lens)
        clock[i] += iteration_seconds(lens)
        kinds = []
        for rid in rids:
            if produced_r[rid] < trace.reasoning[rid]:
                produced_r[rid] += 1
                kinds.append(END_OF_REASONING if produced_r[rid] == trace.reasoning[rid] else TOKEN)
            else:
                produced_a[rid] += 1
                last = produced_a[rid] == trace.answering[rid]
                kinds.append(END_OF_SEQUENCE if last else TOKEN)
                done += last
        ops2 = sched.commit(i, clock[i], kinds)
        log.append(("commit", i, clock[i], tuple(kinds), tuple(ops2)))
        if on_ops:
            on_ops(ops2)
    return log
