"""Priority policy workload (real-time inference preempting best-effort training, latency-weighted timelines;
Sec. 7 of the paper, "Compute-only scheduling" comparison).  CPU part: the driver and the oracle on it."""
import numpy as np
import pytest

from workloads import make_trace, run_priority_schedule
from helpers import check_plan_invariants

NONE = 0xFFFFFFFF


@pytest.mark.parametrize("announce", [False, True])
def test_requests_run_whole_and_best_effort_fills_the_gaps(oracle_mod, announce):
    trace = make_trace(6, scale=32)
    pol = trace.policy
    L, rt, be = pol["request_launches"], pol["rt_task"], pol["be_task"]
    lat = trace.tasks[rt].latency
    assert len({int(x) for x in lat}) > 5                       # profiled latencies, not unit ticks
    o = oracle_mod.Oracle.for_trace(trace)
    done = {rt: 0, be: 0}
    pt_b, fo_b = o.state()
    recs = []
    for rec in run_priority_schedule(trace, o, announce_next_request=announce):
        pt_a, fo_a = o.state()
        check_plan_invariants(rec.plan, pt_b, fo_b, pt_a, fo_a, trace.n_frames)
        pt_b, fo_b = pt_a, fo_a
        assert rec.first_launch == done[rec.task]
        # what the plan covers is resident when it starts
        for g in range(rec.n_launches):
            assert (pt_a[o.command_pages(rec.task, rec.first_launch + g)] != NONE).all()
        if rec.task == rt:
            # the timeline's first entry is exactly the rest of the request
            rest = L - done[rt] % L
            assert rec.timeline[0] == (rt, int(lat[done[rt]:done[rt] + rest].sum()))
            assert rec.plan.g_end0 == rest
        done[rec.task] += rec.n_launches
        recs.append(rec)
    assert done[rt] == len(trace.tasks[rt]) and done[be] == len(trace.tasks[be])
    # a request is never interleaved with best-effort launches
    order = [r.task for r in recs]
    served, i = 0, 0
    while i < len(recs):
        if recs[i].task == rt:
            n = 0
            while n < L:
                assert recs[i].task == rt
                n += recs[i].n_launches
                i += 1
            assert n == L
            served += 1
        else:
            i += 1
    assert served == len(trace.tasks[rt]) // L
    assert be in order and rt in order
    o.close()


def test_a_launch_that_straddles_an_arrival_still_belongs_to_the_gap(oracle_mod):
    trace = make_trace(6, scale=32)
    pol = trace.policy
    o = oracle_mod.Oracle.for_trace(trace)
    be_lat = trace.tasks[pol["be_task"]].latency
    seen = 0
    for rec in run_priority_schedule(trace, o, max_plans=12):
        if rec.task == pol["be_task"] and not rec.replan and rec.plan.covered_launches == rec.plan.g_end0:
            budget = rec.timeline[0][1]
            lats = be_lat[rec.first_launch:rec.first_launch + rec.n_launches].astype(np.int64)
            starts = np.concatenate([[0], np.cumsum(lats)[:-1]])
            assert (starts < budget).all()                      # every launch starts inside the gap
            if rec.first_launch + rec.n_launches < len(be_lat):
                assert starts[-1] + lats[-1] >= budget           # and the next one would not have
            seen += 1
    assert seen >= 2
    o.close()


def test_restoring_the_real_time_working_set_beats_demand_paging(oracle_mod):
    """Pages brought in for the real-time task over the run: the planned migrations against LRU demand paging of
    the same launch order with the same pool."""
    trace = make_trace(6, scale=32)
    o = oracle_mod.Oracle.for_trace(trace)
    planned, order = {0: 0, 1: 0}, []
    for rec in run_priority_schedule(trace, o):
        planned[rec.task] += rec.plan.n_fetch
        order += [(rec.task, rec.first_launch + g) for g in range(rec.n_launches)]
    o.close()
    lru = oracle_mod.Oracle.for_trace(trace)
    from workloads.harness import load_trace
    load_trace(lru, trace)
    faults = lru.lru_faults([t for t, _ in order], [i for _, i in order], trace.n_frames)
    lru.close()
    assert planned[0] + planned[1] < faults
