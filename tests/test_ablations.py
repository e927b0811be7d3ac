"""Ablations of the paper on synthetic schedules (Sec. 5.1 naive allocation-granularity prediction, Sec. 5.2
false negatives with demand paging as the fallback, Sec. 7 Fig. "eval-naive"): CPU part, on the oracle."""
import numpy as np
import pytest

from workloads import make_trace, run_schedule
from workloads.ablation import allocation_granularity, drop_rules
from workloads.harness import load_trace
from helpers import explicit_trace

NONE = 0xFFFFFFFF


def _loaded(oracle_mod, trace, **kw):
    o = oracle_mod.Oracle.for_trace(trace, **kw)
    load_trace(o, trace)
    return o


def _run_with_fallback(oracle_mod, predicted, truth_trace, max_plans=None):
    """Plan from the predicted templates, execute the true launches: what a covered launch really touches and
    does not find resident faults in.  Returns (pages fetched by plans, faults, launches run)."""
    o = _loaded(oracle_mod, predicted)
    truth = _loaded(oracle_mod, truth_trace)
    fetched = faults = launches = 0
    for rec in run_schedule(predicted, o, max_plans=max_plans):
        fetched += rec.plan.n_fetch
        for g in range(rec.n_launches):
            pages = truth.command_pages(rec.task, rec.first_launch + g)
            faults += o.demand_touch(pages)
            pt, fo = o.state()
            assert (pt[pages] != NONE).all()                     # the launch can run
            launches += 1
        res = np.nonzero(pt != NONE)[0]
        assert res.size <= predicted.n_frames and (fo[pt[res]] == res).all()
    o.close()
    truth.close()
    return fetched, faults, launches


def test_allocation_granularity_predicts_a_superset_and_inflates_sparse_buffers(oracle_mod):
    t = make_trace(4, page_shift=15, steps=8, full_backing=True)
    n = allocation_granularity(t)
    a, b = _loaded(oracle_mod, t), _loaded(oracle_mod, n)
    ratio = []
    for task in range(t.n_tasks):
        for i in range(0, len(t.tasks[task]), 7):
            exact, naive = set(a.command_pages(task, i).tolist()), set(b.command_pages(task, i).tolist())
            assert exact <= naive
            ratio.append(len(naive) / len(exact))
    a.close()
    b.close()
    assert max(ratio) > 4                                        # attention launches: weights whole, KV slabs a tenth in use
    assert min(ratio) == 1                                       # weight buffers are touched whole
    # dense training buffers: the naive predictor is exact
    t3 = make_trace(3, scale=32, iterations=2)
    n3 = allocation_granularity(t3)
    a, b = _loaded(oracle_mod, t3), _loaded(oracle_mod, n3)
    for i in range(0, len(t3.tasks[0]), 5):
        assert np.array_equal(a.command_pages(0, i), b.command_pages(0, i))
    a.close()
    b.close()


def test_migration_volume_inflates_under_the_naive_predictor(oracle_mod):
    t = make_trace(4, page_shift=15, steps=16, full_backing=True)
    vol = {}
    for name, tr in (("template", t), ("allocation", allocation_granularity(t))):
        o = _loaded(oracle_mod, tr)
        vol[name] = sum(rec.plan.n_fetch for rec in run_schedule(tr, o))
        o.close()
    assert vol["allocation"] > 4 * vol["template"], vol         # the paper reports 4.8x to 12x


def test_perfect_prediction_never_faults(oracle_mod):
    t = make_trace(3, scale=32, iterations=2)
    fetched, faults, launches = _run_with_fallback(oracle_mod, t, t)
    assert faults == 0 and launches == t.total_launches() and fetched > 0


def test_false_negatives_fault_in_and_the_run_completes(oracle_mod):
    t = make_trace(3, scale=32, iterations=3)
    seen = []
    for rate in (0.0025, 0.02, 0.2):
        fetched, faults, launches = _run_with_fallback(oracle_mod, drop_rules(t, rate, seed=1), t)
        assert launches == t.total_launches()
        seen.append(faults)
    assert 0 < seen[0] < seen[1] < seen[2]
    exact = sum(rec.plan.n_fetch for rec in run_schedule(t, _loaded(oracle_mod, t)))
    assert seen[0] < 0.02 * exact                                # at the paper's 0.25 % the fallback is noise


def test_a_fault_evicts_the_page_needed_farthest_in_the_future(oracle_mod):
    # one task, pool of 4 frames; launches touch {0,1}, {2}, {3}, then {0,1} again; page 7 is never predicted
    trace = explicit_trace([[[0, 1], [2], [3], [0, 1]]], 8, 4, timeslice=4)
    o = _loaded(oracle_mod, trace)
    plan = o.plan([(0, 4)])
    assert plan.covered_launches == 4 and plan.n_fetch == 4
    o.migrate()
    pt, _ = o.state()
    assert (pt[[0, 1, 2, 3]] != NONE).all()
    # launch 0 really touches {0, 1, 7}: 7 faults; next uses are 0:0 1:0 2:1 3:2 -> page 3 is the farthest
    assert o.demand_touch([0, 1, 7]) == 1
    pt, fo = o.state()
    assert pt[3] == NONE and pt[7] != NONE and (pt[[0, 1, 2]] != NONE).all()
    # touching resident pages costs nothing; a second miss takes the next farthest, page 2 (7 is in use now)
    assert o.demand_touch([0, 1, 7]) == 0
    assert o.demand_touch([5, 7]) == 1
    pt, _ = o.state()
    assert pt[2] == NONE and pt[5] != NONE and pt[7] != NONE
    # pages in use by the faulting launch are never its victims
    assert o.demand_touch([0, 1, 5, 6]) == 1
    pt, _ = o.state()
    assert pt[7] == NONE and (pt[[0, 1, 5, 6]] != NONE).all()
    with pytest.raises(oracle_mod.OracleError):
        o.demand_touch([0, 1, 2, 3, 4])                         # more pages than frames
    o.close()
