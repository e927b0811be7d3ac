"""Pins for the oracle's placement policy (Sec. 6.1-6.2 of the paper: OPT / Belady
eviction order resolved from the task timeline).  Expected values come from
independent computations written here: exhaustive search over all eviction
choices, textbook MIN over a flat reference string, the paper's three-task
eviction-order example, and a steady state derived by hand."""
import itertools
from functools import lru_cache

import numpy as np
import pytest

from workloads import make_trace, run_schedule
from workloads.harness import load_trace
from helpers import explicit_trace, check_plan_invariants

NONE = 0xFFFFFFFF


def _run(oracle_mod, trace, horizon="round", with_bytes=False, check=True, max_plans=None):
    o = oracle_mod.Oracle.for_trace(trace, with_bytes=with_bytes)
    load_trace(o, trace)
    recs = []
    pt0, fo0 = o.state()
    for rec in run_schedule(trace, o, horizon=horizon, max_plans=max_plans):
        pt1, fo1 = o.state()
        if check:
            check_plan_invariants(rec.plan, pt0, fo0, pt1, fo1, trace.n_frames)
            # every page of every launch that is about to run is resident
            for i in range(rec.first_launch, rec.first_launch + rec.n_launches):
                assert (pt1[o.command_pages(rec.task, i)] != NONE).all()
        pt0, fo0 = pt1, fo1
        recs.append(rec)
    return o, recs


def _optimal_fetches(wsets, n_frames):
    """Minimum total pages fetched over every possible choice of victims (any subset of
    the resident pages outside the working set, over-eviction allowed) at every switch."""
    wsets = [frozenset(w) for w in wsets]

    @lru_cache(maxsize=None)
    def best(s, resident):
        if s == len(wsets):
            return 0
        w = wsets[s]
        fetch = w - resident
        others = sorted(resident - w)
        need = max(0, len(resident) + len(fetch) - n_frames)
        out = None
        for k in range(need, len(others) + 1):
            for ev in itertools.combinations(others, k):
                c = best(s + 1, (resident - frozenset(ev)) | w)
                out = c if out is None else min(out, c)
        return len(fetch) + out

    return best(0, frozenset())


def test_full_horizon_plans_fetch_the_exhaustive_minimum(oracle_mod):
    rng = np.random.default_rng(11)
    checked = 0
    for trial in range(120):
        n_tasks = int(rng.integers(2, 4))
        n_pages = int(rng.integers(5, 9))
        n_frames = int(rng.integers(4, 6))
        slice_len = int(rng.integers(1, 3))
        cmds = [[sorted(rng.choice(n_pages, size=int(rng.integers(1, 3)), replace=False).tolist())
                 for _ in range(int(rng.integers(2, 5)))] for _ in range(n_tasks)]
        trace = explicit_trace(cmds, n_pages, n_frames, slice_len)
        o, recs = _run(oracle_mod, trace, horizon="full")
        if any(r.replan for r in recs):
            continue
        wsets = [set().union(*[cmds[r.task][i] for i in range(r.first_launch, r.first_launch + r.n_launches)])
                 for r in recs]
        got = sum(r.plan.n_fetch for r in recs)
        assert got == _optimal_fetches(wsets, n_frames), (trial, cmds, n_frames, slice_len)
        checked += 1
    assert checked > 80


def _textbook_min_misses(refs, capacity):
    """Belady's MIN on a reference string: on a miss with a full cache evict the page
    whose next reference is farthest in the future (never = farthest)."""
    cache, misses = set(), 0
    for i, p in enumerate(refs):
        if p in cache:
            continue
        misses += 1
        if len(cache) == capacity:
            def next_ref(q):
                for j in range(i + 1, len(refs)):
                    if refs[j] == q:
                        return j
                return len(refs) + 1
            cache.remove(max(cache, key=next_ref))
        cache.add(p)
    return misses


def test_one_page_commands_reduce_to_textbook_min(oracle_mod):
    rng = np.random.default_rng(5)
    for trial in range(60):
        n_tasks, n_pages = int(rng.integers(1, 4)), int(rng.integers(4, 12))
        n_frames = int(rng.integers(2, 5))
        cmds = [[[int(rng.integers(0, n_pages))] for _ in range(int(rng.integers(3, 12)))]
                for _ in range(n_tasks)]
        trace = explicit_trace(cmds, n_pages, n_frames, timeslice=1)
        o, recs = _run(oracle_mod, trace, horizon="full")
        refs = [cmds[r.task][r.first_launch][0] for r in recs]
        assert sum(r.plan.n_fetch for r in recs) == _textbook_min_misses(refs, n_frames)


def _read_golden(name):
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)
    out = {}
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            key, val = line.split(":", 1)
            out[key.strip()] = val.strip()
    return out


def test_three_task_example_eviction_order(oracle_mod):
    """Sec. 6.2, memory-manager figure (tests/golden/sec6_2_three_task_timeline.txt): with the
    timeline Task1 (20 ms) -> Task2 (10 ms) -> Task3 (30 ms), the eviction order is: pages
    unreferenced across the timeline, then Task3's working set, then Task2's, then Task1's; migrate
    populates Task1's set."""
    gold = _read_golden("sec6_2_three_task_timeline.txt")
    ms = int(gold["command_ms"])
    cmds_of = lambda key: [[int(x) for x in part.split()] for part in gold[key].split("|")]
    t1, t2, t3, idle = cmds_of("task1"), cmds_of("task2"), cmds_of("task3"), cmds_of("idle")
    tl = [int(x) for x in gold["timeline"].split()]
    timeline = [(tl[i] - 1, tl[i + 1]) for i in range(0, len(tl), 2)]     # tasks are numbered from 1 in the paper
    assert gold["eviction_class_order"].split() == ["idle", "task3", "task2", "task1"]
    cmds = [t1, t2, t3, idle]
    lat = [[ms] * len(c) for c in cmds]
    trace = explicit_trace(cmds, 48, 16, timeslice=20, latencies=lat)
    o = oracle_mod.Oracle.for_trace(trace)
    load_trace(o, trace)
    # bring the idle task's, Task3's and Task2's slices into HBM (16 frames: 6 + 6 + 4)
    for warm in ([(3, 20)], [timeline[2]], [timeline[1]]):
        p = o.plan(warm)
        assert p.n_evict == 0
        o.migrate()
    o.launch_retire(3, 2)                        # the idle task has nothing queued any more
    p = o.plan(timeline)
    assert (p.g_end0, p.g_cut, p.n_commands) == (2, 2, 6)
    assert p.fetch_pages.tolist() == [q for c in t1 for q in c]     # Task1's set, in access order
    assert p.n_free_used == 0 and p.n_evict == 8
    ev = p.evict_pages.tolist()
    idle_pages = sorted(q for c in idle for q in c)
    assert ev[:6] == idle_pages                                     # unreferenced first
    assert ev[6:] == t3[2]                                          # then the far end of Task3's slice
    assert not set(ev) & set(q for c in t2 for q in c)              # Task2's and Task1's classes are not reached


def test_victims_come_class_by_class_unreferenced_then_farthest_slice(oracle_mod):
    """Same example, pool so small that the victims span all three classes."""
    ms = 10
    grey = [[40, 41]]
    t1 = [[0, 1, 2, 3], [4, 5, 6, 7]]
    t2 = [[10, 11, 12, 13]]
    t3 = [[20, 21], [22, 23], [24, 25]]
    cmds = [t1, t2, t3, grey]
    lat = [[ms] * len(c) for c in cmds]
    trace = explicit_trace(cmds, 48, 12, timeslice=20, latencies=lat)
    o = oracle_mod.Oracle.for_trace(trace)
    load_trace(o, trace)
    for tl in ([(3, 10)], [(2, 30)], [(1, 10)]):
        o.plan(tl)
        o.migrate()
    o.launch_retire(3, 1)
    p = o.plan([(0, 20), (1, 10), (2, 30)])
    # 12 frames hold grey(2) + Task3(6) + Task2(4); Task1 needs 8: all grey, all of Task3 ... in order
    assert p.n_evict == 8
    assert p.evict_pages.tolist() == [40, 41, 24, 25, 22, 23, 20, 21]
    assert p.fetch_frames.tolist() == p.evict_frames.tolist()
    # one more page needed -> the first page of Task2's set goes next
    trace2 = explicit_trace([[[0, 1, 2, 3], [4, 5, 6, 7]], [[10, 11, 12, 13]],
                             [[20, 21], [22, 23], [24, 25]], [[40]]], 48, 11, 20, latencies=[[ms] * 2, [ms], [ms] * 3, [ms]])
    o = oracle_mod.Oracle.for_trace(trace2)
    load_trace(o, trace2)
    for tl in ([(3, 10)], [(2, 30)], [(1, 10)]):
        o.plan(tl)
        o.migrate()
    o.launch_retire(3, 1)
    p = o.plan([(0, 20), (1, 10), (2, 30)])
    assert p.evict_pages.tolist() == [40, 24, 25, 22, 23, 20, 21, 10]


def test_pool_at_least_footprint_never_evicts(oracle_mod):
    trace = make_trace(1, seed=3)
    trace.n_frames = trace.n_virtual_pages
    o, recs = _run(oracle_mod, trace)
    assert all(r.plan.n_evict == 0 for r in recs)
    touched = set()
    for t, cmds in enumerate(trace.tasks):
        for i in range(len(cmds)):
            touched |= set(o.command_pages(t, i).tolist())
    fetched = np.concatenate([r.plan.fetch_pages for r in recs])
    assert fetched.size == len(touched) and set(fetched.tolist()) == touched


def test_stencil_sweep_steady_state_closed_form(oracle_mod):
    """4 tasks x 384 pages, every launch touches all of its task's pages, 1024 frames, one
    round of look-ahead.  By hand: the first four switches fetch 384 each (the third evicts
    128, the fourth 384); after that (fetch, evict) repeats (0,0), (128,128), (384,384).
    80 switches fetch 4*384 + 25*512 = 14336 pages.  LRU on the same trace misses every page
    of every slice: 80 * 384 = 30720."""
    trace = make_trace(2, page_shift=12)
    o, recs = _run(oracle_mod, trace, check=False)
    assert len(recs) == 80
    pairs = [(r.plan.n_fetch, r.plan.n_evict) for r in recs]
    assert pairs[:4] == [(384, 0), (384, 0), (384, 128), (384, 384)]
    cycle = [(0, 0), (128, 128), (384, 384)]
    assert pairs[4:] == [cycle[i % 3] for i in range(76)]
    assert sum(p[0] for p in pairs) == 14336
    tasks, idx = [], []
    for r in recs:
        tasks += [r.task] * r.n_launches
        idx += list(range(r.first_launch, r.first_launch + r.n_launches))
    assert o.lru_faults(tasks, idx, trace.n_frames) == 30720


def test_eviction_takes_only_what_is_needed_and_never_prefetches(oracle_mod):
    trace = make_trace(1, seed=1)
    o, recs = _run(oracle_mod, trace)
    for r in recs:
        covered = set()
        for i in range(r.first_launch, r.first_launch + r.n_launches):
            covered |= set(o.command_pages(r.task, i).tolist())
        assert set(r.plan.fetch_pages.tolist()) <= covered      # nothing of later slices is fetched


@pytest.mark.parametrize("cfg,kw", [
    (1, dict(seed=0)), (1, dict(seed=5)),
    (3, dict(scale=64, layers=6, iterations=3)),
    (4, dict(page_shift=12, layers=4, steps=12)),
    (5, dict(scale=256, n_launches=20)),
])
def test_invariants_hold_on_every_schedule(oracle_mod, cfg, kw):
    trace = make_trace(cfg, **kw)
    o, recs = _run(oracle_mod, trace)
    assert sum(r.n_launches for r in recs) == trace.total_launches()
    for r in recs:                      # fetch list is in order of use, then page id
        assert r.plan.covered_launches >= 1


def test_oversized_slice_is_cut_to_a_fitting_prefix(oracle_mod):
    # 6 frames: commands 0 and 1 together need 8 pages, so only the first is covered;
    # the re-plan covers commands 1 and 2 (6 distinct pages)
    trace = explicit_trace([[[0, 1, 2, 3], [4, 5, 6, 7], [0, 1, 4, 5]]], 8, 6, timeslice=3)
    o, recs = _run(oracle_mod, trace)
    assert [(r.plan.g_end0, r.plan.covered_launches, r.replan) for r in recs] == [(3, 1, False), (2, 2, True)]
    # a single command larger than the pool cannot be served
    trace = explicit_trace([[[0, 1, 2, 3]]], 8, 3, timeslice=1)
    o = oracle_mod.Oracle.for_trace(trace)
    load_trace(o, trace)
    with pytest.raises(oracle_mod.OracleError) as e:
        o.plan([(0, 1)])
    assert e.value.name == "E_WSET_TOO_LARGE"
    # an empty timeline or an idle task plans nothing
    p = o.plan([])
    assert (p.n_fetch, p.n_evict, p.covered_launches) == (0, 0, 0)


def test_latency_decides_which_commands_fall_in_a_slice(oracle_mod):
    # latencies 3,3,3: a 7-tick slice starts three commands (0,3,6 < 7), a 6-tick slice two
    trace = explicit_trace([[[0], [1], [2], [3]]], 8, 8, timeslice=7, latencies=[[3, 3, 3, 3]])
    o = oracle_mod.Oracle.for_trace(trace)
    load_trace(o, trace)
    assert o.plan([(0, 7)]).fetch_pages.tolist() == [0, 1, 2]
    assert o.plan([(0, 6)]).fetch_pages.tolist() == [0, 1]
    assert o.plan([(0, 1)]).fetch_pages.tolist() == [0]
    # a task listed twice continues where its first entry stopped
    p = o.plan([(0, 3), (0, 6)])
    assert (p.g_end0, p.n_commands) == (1, 3)


def _list_lru_faults(refs, capacity):
    """LRU as the textbooks state it: a recency list, most recent last."""
    order, faults = [], 0
    for p in refs:
        if p in order:
            order.remove(p)
        else:
            faults += 1
            if len(order) == capacity:
                order.pop(0)
        order.append(p)
    return faults


def test_lru_simulator_is_textbook_lru(oracle_mod):
    """The demand-paging baseline (Sec. 6.2 "Driver support": a fault with full HBM evicts from the head of the
    driver's LRU list).  A capacity of exactly n frames: n distinct pages cycled forever miss n times, n + 1
    distinct pages cycled miss every time; random reference strings agree with a recency-list LRU."""
    for n in (1, 2, 3, 7):
        cyc = [[[p] for _ in range(5) for p in range(n)]]
        trace = explicit_trace(cyc, n + 1, n, timeslice=1)
        o = oracle_mod.Oracle.for_trace(trace)
        load_trace(o, trace)
        assert o.lru_faults([0] * (5 * n), list(range(5 * n)), n) == n
        o.close()
        cyc = [[[p] for _ in range(5) for p in range(n + 1)]]
        trace = explicit_trace(cyc, n + 1, n, timeslice=1)
        o = oracle_mod.Oracle.for_trace(trace)
        load_trace(o, trace)
        assert o.lru_faults([0] * (5 * (n + 1)), list(range(5 * (n + 1))), n) == 5 * (n + 1)
        o.close()
    rng = np.random.default_rng(11)
    for trial in range(40):
        n_pages, cap = int(rng.integers(3, 14)), int(rng.integers(1, 6))
        refs = [int(x) for x in rng.integers(0, n_pages, int(rng.integers(5, 60)))]
        trace = explicit_trace([[[p] for p in refs]], n_pages, max(cap, 1), timeslice=1)
        o = oracle_mod.Oracle.for_trace(trace)
        load_trace(o, trace)
        assert o.lru_faults([0] * len(refs), list(range(len(refs))), cap) == _list_lru_faults(refs, cap)
        o.close()
