"""Small trace builders and independent reference computations used by the tests."""
import numpy as np

from workloads import Rule, Trace, RULE_FIXED
from workloads.trace import CommandBuilder


def explicit_trace(task_cmds, n_pages, n_frames, timeslice, page_shift=8, latencies=None, name="explicit"):
    """task_cmds[t][i] = iterable of page ids touched by launch i of task t (at most 4 each).
    Every launch uses kernel k with k one-page FIXED rules, so its page set is exactly the ids given."""
    P = 1 << page_shift
    kernels = [[Rule(RULE_FIXED, r, (), P) for r in range(k)] for k in range(5)]
    tasks = []
    for t, cmds in enumerate(task_cmds):
        b = CommandBuilder()
        for i, pages in enumerate(cmds):
            pages = list(pages)
            assert len(pages) <= 4
            lat = 1 if latencies is None else latencies[t][i]
            b.add(len(pages), [p * P for p in pages], latency=lat)
        tasks.append(b.build())
    return Trace(name=name, page_shift=page_shift, n_virtual_pages=n_pages, n_frames=n_frames,
                 timeslice=timeslice, kernels=kernels, tasks=tasks, n_slots=n_pages)


def check_plan_invariants(plan, pt_before, fo_before, pt_after, fo_after, n_frames):
    """Properties every plan + migrate must satisfy, whatever the policy's tie-breaks."""
    NONE = 0xFFFFFFFF
    n_free = int((fo_before == NONE).sum())
    assert plan.n_evict == max(0, plan.n_fetch - n_free)
    assert plan.n_free_used == min(n_free, plan.n_fetch)
    assert len(set(plan.fetch_pages.tolist())) == plan.n_fetch
    assert len(set(plan.evict_pages.tolist())) == plan.n_evict
    assert not set(plan.fetch_pages.tolist()) & set(plan.evict_pages.tolist())
    assert (pt_before[plan.fetch_pages] == NONE).all()
    assert (pt_before[plan.evict_pages] == plan.evict_frames).all()
    assert (pt_after[plan.evict_pages] == NONE).all()
    assert (pt_after[plan.fetch_pages] == plan.fetch_frames).all()
    assert len(set(plan.fetch_frames.tolist())) == plan.n_fetch
    resident = np.nonzero(pt_after != NONE)[0]
    assert resident.size <= n_frames
    assert (fo_after[pt_after[resident]] == resident).all()
    owned = np.nonzero(fo_after != NONE)[0]
    assert owned.size == resident.size
    assert (pt_after[fo_after[owned]] == owned).all()
