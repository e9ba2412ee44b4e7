"""TEST INFRASTRUCTURE ONLY: replay of request arranging across arrivals on the CPU.

The paper (Section 4.2, "Request arranging") places a new request behind the queued requests of the same expert, so
that they run as one group and the expert is loaded at most once for all of them.  Requests can only meet in the
queue if a small group is allowed to wait there; this module replays that waiting rule, step by step, for a given
arrival sequence and the routes the chain oracle computed, and drives the expert-cache replay (Sections 4.1, 4.3)
with the groups that actually run.  Everything here is integer bookkeeping: it fixes WHICH requests run in WHICH
step and which switches that causes, never a numerical result (those do not depend on the schedule).

The waiting rule, per queued group of expert e at step k:
    age    = k - (number of the first step that saw the group's oldest request)
    enough = min_resident(arch of e) if e is on the device at the start of the step, else min_missing(arch of e)
    the group stays queued  iff  age < max_wait(arch of e)  and  size < enough
The thresholds come from the latency model of Section 4.2 (a batch of n requests of one expert takes K n + B, a
missing expert adds its load time): a group is worth running once the fixed part per request is small.

Also here: the rule that gives units of work to parallel executors ("Request assigning").

Pinned by tests/test_oracle_routing.py: a hand-worked schedule, invariants on random arrival sequences (nobody waits
longer than max_wait, every request runs every stage of its path exactly once and in order), reduction to the
window-less schedule for max_wait = 0; a hand-worked assignment."""
from typing import Dict, List, Optional, Sequence, Tuple


def stays_queued(size: int, age: int, resident: bool, min_resident: int, min_missing: int, max_wait: int) -> bool:
    if size <= 0 or age >= max_wait:
        return False
    return size < (min_resident if resident else min_missing)


def replay(submits: Sequence[Sequence[int]], paths: Sequence[Sequence[int]], arch_of: Sequence[int],
           window: Dict[int, Tuple[int, int, int]], cache=None, max_steps: int = 100000) -> List[dict]:
    """submits[k]: the requests handed over right before the k-th step (k counts the steps that found something
    queued); after the last hand-over, steps go on until the queue is empty.  paths[r]: the experts request r visits,
    in order (from the chain oracle).  arch_of[e]: architecture of expert e; window[arch] = (min_resident,
    min_missing, max_wait), a missing arch means no window.  cache: an oracle.CacheSim already past its initial fill
    (None: every expert counts as resident and nothing is ever switched).

    Returns one record per step: dict(step, n_pending, run={expert: [requests...]}, deferred={expert: [requests...]},
    order=[experts in execution order], switches=[(expert, [victims...])...])."""
    n_experts = len(arch_of)
    pos = {}            # request -> index into its path of the stage it is queued for
    first_seen = {}     # request -> number of the first step that saw it
    records = []
    step = 0
    hand = 0
    while True:
        if hand < len(submits):
            for r in submits[hand]:
                r = int(r)
                assert r not in first_seen, "request submitted twice"
                pos[r] = 0
                first_seen[r] = step
            hand += 1
        if not pos:
            if hand >= len(submits):
                break
            continue                      # an empty probing step does not count
        assert step < max_steps, "the queue does not drain"
        groups: Dict[int, List[int]] = {}
        for r in sorted(pos):
            groups.setdefault(int(paths[r][pos[r]]), []).append(r)
        resident = cache.resident() if cache is not None else [True] * n_experts
        run, deferred = {}, {}
        for e, members in groups.items():
            mr, mm, mw = window.get(int(arch_of[e]), (0, 0, 0))
            age = step - min(first_seen[r] for r in members)
            (deferred if stays_queued(len(members), age, bool(resident[e]), mr, mm, mw) else run)[e] = members
        has_group = [e in run for e in range(n_experts)]
        if cache is not None:
            order, switches = cache.stage(has_group)
        else:
            order, switches = sorted(run), []
        assert sorted(order) == sorted(run)
        records.append(dict(step=step, n_pending=sum(len(m) for m in groups.values()), run=run, deferred=deferred,
                            order=order, switches=switches))
        for members in run.values():
            for r in members:
                pos[r] += 1
                if pos[r] == len(paths[r]):
                    del pos[r]
        step += 1
    return records


def assign(costs: Sequence[int], n_executors: int) -> List[int]:
    """Request assigning (paper Section 4.2): executors work in parallel, the total time is that of the longest queue,
    and a new unit of work goes where that total stays smallest; among queues that tie, to the one whose own time
    grows to the smallest value.  For equal executors both criteria pick a queue with the least work so far; the
    lowest-numbered one is taken.  costs: predicted cost of the units in arrival order.  Returns the executor of each."""
    assert n_executors >= 1
    queue_time = [0] * n_executors
    out = []
    for cst in costs:
        totals = []
        for q in range(n_executors):
            after = list(queue_time)
            after[q] += int(cst)
            totals.append((max(after), after[q], q))        # total time, this queue's time, index
        q = min(totals)[2]
        queue_time[q] += int(cst)
        out.append(q)
    return out
