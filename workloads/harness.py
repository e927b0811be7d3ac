"""Round-robin driver: plays the scheduler that calls the memory manager at
every context switch (Sec. 6.1 of the paper) against any implementation that
offers the calls below.  It builds timelines and retires launches; it never
looks at pages.

Implementation protocol (duck-typed; the oracle wrapper and the HIP binding
both satisfy it):
    kernel_register(rules) -> kernel id
    task_create() -> task id
    launch_enqueue(task, kernel_id, args_u64, n_args, latency, ids_off, n_ids)
    launch_retire(task, n)
    plan(timeline) -> object with n_fetch, n_evict, n_free_used, g_cut, g_end0,
                      covered_launches
    migrate()
"""
from dataclasses import dataclass
from typing import Iterator, List, Optional, Tuple

import numpy as np

from .trace import Trace


@dataclass
class SwitchRecord:
    index: int                       # running count of plan calls
    task: int                        # incoming task
    timeline: List[Tuple[int, int]]  # (task, timeslice ticks) entries passed to plan
    plan: object                     # what impl.plan returned
    first_launch: int                # index (in the task's program order) of the first covered launch
    n_launches: int                  # launches that run before the next plan call
    replan: bool                     # True when the previous plan was truncated


def load_trace(impl, trace: Trace) -> None:
    """Register templates and enqueue every launch up front (launches are
    asynchronous and run far ahead of execution)."""
    kid = [impl.kernel_register(rules) for rules in trace.kernels]
    for t, cmds in enumerate(trace.tasks):
        tid = impl.task_create()
        assert tid == t
        for i in range(len(cmds)):
            impl.launch_enqueue(t, kid[int(cmds.kernel_id[i])], cmds.args[i], int(cmds.n_args[i]),
                                int(cmds.latency[i]), int(cmds.ids_off[i]), int(cmds.n_ids[i]))


def _slice_count(latency: np.ndarray, start: int, ticks: int) -> int:
    """Launches of one task, from `start`, that begin inside a timeslice of `ticks`."""
    acc, n = 0, 0
    while start + n < latency.shape[0] and acc < ticks:
        acc += int(latency[start + n])
        n += 1
    return n


def _timeline(trace: Trace, cursor: List[int], cur: int, first_ticks: int, horizon: str):
    n = trace.n_tasks
    remaining = [len(trace.tasks[t]) - cursor[t] for t in range(n)]
    entries = []
    if horizon == "round":
        for k in range(n):
            t = (cur + k) % n
            if remaining[t] > 0:
                entries.append((t, first_ticks if k == 0 else trace.timeslice))
        return entries
    # full horizon: the whole remaining round-robin schedule
    pos = list(cursor)
    t, ticks = cur, first_ticks
    while any(pos[i] < len(trace.tasks[i]) for i in range(n)):
        if pos[t] < len(trace.tasks[t]):
            entries.append((t, ticks))
            pos[t] += _slice_count(trace.tasks[t].latency, pos[t], ticks)
        t, ticks = (t + 1) % n, trace.timeslice
    return entries


class LazyLoader:
    """Enqueues launches a bounded distance ahead of execution instead of all up front: new
    commands keep arriving between context switches (training loops, decoding; Sec. 6.2 of the
    paper on dynamically launched commands), and queues shrink and grow as launches retire."""

    def __init__(self, impl, trace: Trace, ahead_slices: int = 3):
        self.impl, self.trace = impl, trace
        self.kid = [impl.kernel_register(rules) for rules in trace.kernels]
        self.sent = [0] * trace.n_tasks
        self.ahead = ahead_slices
        for t in range(trace.n_tasks):
            assert impl.task_create() == t

    def top_up(self, cursor):
        """Make sure every task has its next `ahead` timeslices queued."""
        for t, cmds in enumerate(self.trace.tasks):
            want = cursor[t]
            for _ in range(self.ahead):
                want += _slice_count(cmds.latency, want, self.trace.timeslice)
            while self.sent[t] < want:
                i = self.sent[t]
                self.impl.launch_enqueue(t, self.kid[int(cmds.kernel_id[i])], cmds.args[i], int(cmds.n_args[i]),
                                         int(cmds.latency[i]), int(cmds.ids_off[i]), int(cmds.n_ids[i]))
                self.sent[t] += 1


def run_schedule(trace: Trace, impl, horizon: str = "round", max_plans: Optional[int] = None,
                 loader: Optional[LazyLoader] = None) -> Iterator[SwitchRecord]:
    """Drive `impl` through the trace.  Yields after each plan + migrate and
    before the covered launches are retired, so the caller can inspect state
    at the moment those launches would start.  With a `loader`, launches are
    enqueued only a few timeslices ahead (one round of look-ahead must fit)."""
    n = trace.n_tasks
    cursor = [0] * n
    cur, index = 0, 0
    while any(cursor[t] < len(trace.tasks[t]) for t in range(n)):
        if loader is not None:
            loader.top_up(cursor)
        if cursor[cur] >= len(trace.tasks[cur]):
            cur = (cur + 1) % n
            continue
        budget, replan = trace.timeslice, False
        while budget > 0 and cursor[cur] < len(trace.tasks[cur]):
            if loader is not None:
                loader.top_up(cursor)
            tl = _timeline(trace, cursor, cur, budget, horizon)
            plan = impl.plan(tl)
            impl.migrate()
            covered = int(plan.covered_launches)
            yield SwitchRecord(index, cur, tl, plan, cursor[cur], covered, replan)
            index += 1
            lat = trace.tasks[cur].latency
            budget -= int(lat[cursor[cur]:cursor[cur] + covered].sum())
            impl.launch_retire(cur, covered)
            cursor[cur] += covered
            if max_plans is not None and index >= max_plans:
                return
            if covered == int(plan.g_end0):
                break
            replan = True
        cur = (cur + 1) % n


def run_priority_schedule(trace: Trace, impl, max_plans: Optional[int] = None,
                          announce_next_request: bool = False) -> Iterator[SwitchRecord]:
    """Priority policy (Sec. 7 of the paper, real-time beside best-effort): the real-time task's requests
    arrive every `period` ticks, preempt the best-effort task at its next launch boundary and run to
    completion; the best-effort task runs in the gaps.  A request's launches are enqueued when it arrives
    (dynamically launched commands), or, with announce_next_request, as soon as the previous request has
    finished, so that plans made for the best-effort task already see the next request in the timeline.
    `impl` must be empty: kernels, tasks and launches are registered here.  Time is counted in ticks of
    profiled latency; a launch belongs to the slice it starts in, so the one that straddles an arrival
    delays the request by its remainder."""
    pol = trace.policy
    rt, be, L, period = pol["rt_task"], pol["be_task"], pol["request_launches"], pol["period"]
    kid = [impl.kernel_register(rules) for rules in trace.kernels]
    for t in range(trace.n_tasks):
        assert impl.task_create() == t

    def enqueue(t, lo, hi):
        cmds = trace.tasks[t]
        for i in range(lo, hi):
            impl.launch_enqueue(t, kid[int(cmds.kernel_id[i])], cmds.args[i], int(cmds.n_args[i]),
                                int(cmds.latency[i]), int(cmds.ids_off[i]), int(cmds.n_ids[i]))

    n_be, n_req = len(trace.tasks[be]), len(trace.tasks[rt]) // L
    enqueue(be, 0, n_be)
    lat = {t: trace.tasks[t].latency.astype(np.int64) for t in (rt, be)}
    cursor = {rt: 0, be: 0}
    sent, now, req, index = 0, 0, 0, 0

    def step(task, tl, replan):
        nonlocal index, now
        plan = impl.plan(tl)
        impl.migrate()
        covered = int(plan.covered_launches)
        rec = SwitchRecord(index, task, tl, plan, cursor[task], covered, replan)
        index += 1
        now += int(lat[task][cursor[task]:cursor[task] + covered].sum())
        return rec, covered

    if announce_next_request and n_req:
        enqueue(rt, 0, L)
        sent = L
    while req < n_req or cursor[be] < n_be:
        arrival = req * period
        if req < n_req and now >= arrival:                     # a request runs to completion
            if sent < (req + 1) * L:
                enqueue(rt, sent, (req + 1) * L)
                sent = (req + 1) * L
            replan = False
            while cursor[rt] < (req + 1) * L:
                ticks = int(lat[rt][cursor[rt]:(req + 1) * L].sum())
                tl = [(rt, ticks)]
                if cursor[be] < n_be:
                    tl.append((be, max(1, (req + 1) * period - now - ticks)))
                rec, covered = step(rt, tl, replan)
                yield rec
                impl.launch_retire(rt, covered)
                cursor[rt] += covered
                replan = True
                if max_plans is not None and index >= max_plans:
                    return
            req += 1
            if announce_next_request and req < n_req:
                enqueue(rt, sent, (req + 1) * L)
                sent = (req + 1) * L
        elif cursor[be] < n_be:                                # the best-effort task fills the gap
            budget = (arrival - now) if req < n_req else pol["be_quantum"]
            replan = False
            while budget > 0 and cursor[be] < n_be:
                tl = [(be, budget)]
                if req < n_req:
                    tl.append((rt, trace.timeslice))           # holds commands only once the request is known
                    tl.append((be, period))
                before = now
                rec, covered = step(be, tl, replan)
                yield rec
                impl.launch_retire(be, covered)
                cursor[be] += covered
                budget -= now - before
                if max_plans is not None and index >= max_plans:
                    return
                if covered == int(rec.plan.g_end0):
                    break
                replan = True
        else:
            now = arrival                                      # idle until the next request
