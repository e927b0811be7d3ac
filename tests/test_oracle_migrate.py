"""Pins for the oracle's migration step (Sec. 6.2 "Driver support", Sec. 6.3) and its
LRU demand-paging simulator.  Page bytes are a fixed function of (page, word), the
running task overwrites one word of every page it brought in, and after any number
of switches every page must read back unchanged from wherever it lives."""
import numpy as np

from workloads import make_trace, run_schedule, page_words, stamp_of
from workloads.harness import load_trace
from helpers import explicit_trace

NONE = 0xFFFFFFFF


def _round_trip(oracle_mod, trace, max_plans=None):
    o = oracle_mod.Oracle.for_trace(trace, with_bytes=True)
    load_trace(o, trace)
    wpp = trace.page_bytes // 8
    pages_with_slot = (np.arange(trace.n_virtual_pages) if trace.host_slot is None
                       else np.nonzero(trace.host_slot != NONE)[0])
    truth = np.zeros((trace.n_virtual_pages, wpp), np.uint64)
    truth[pages_with_slot] = page_words(pages_with_slot, wpp)
    o.host_words[o.slot_of(pages_with_slot)] = truth[pages_with_slot]
    o.pool_words[:] = np.uint64(0xDEADBEEFDEADBEEF)
    moved = 0
    for rec in run_schedule(trace, o, max_plans=max_plans):
        pl = rec.plan
        # the task now running writes one word into every page that was just brought in
        idx, val = stamp_of(pl.fetch_pages, rec.index, wpp)
        o.pool_words[pl.fetch_frames, idx] = val
        truth[pl.fetch_pages, idx] = val
        moved += pl.n_fetch + pl.n_evict
        pt, fo = o.state()
        res = np.nonzero(pt != NONE)[0]
        assert np.array_equal(o.pool_words[pt[res]], truth[res])
        out = np.setdiff1d(pages_with_slot, res)
        assert np.array_equal(o.host_words[o.slot_of(out)], truth[out])
    return moved


def test_contents_survive_round_trips_tiny(oracle_mod):
    assert _round_trip(oracle_mod, make_trace(1, seed=0, page_shift=11)) > 1000


def test_contents_survive_round_trips_sparse_backing_store(oracle_mod):
    assert _round_trip(oracle_mod, make_trace(4, page_shift=8, layers=3, steps=10)) > 500


def test_eviction_writes_back_what_the_task_wrote(oracle_mod):
    # 2 frames, pages 0,1 then 2,3 then 0,1 again: the stamp written while 0,1 were resident
    # must come back from the host copy
    trace = explicit_trace([[[0, 1], [2, 3], [0, 1]]], 4, 2, timeslice=1, page_shift=6)
    o = oracle_mod.Oracle.for_trace(trace, with_bytes=True)
    load_trace(o, trace)
    wpp = 8
    o.host_words[:] = page_words(np.arange(4), wpp)
    p = o.plan([(0, 1)]); o.migrate(); o.launch_retire(0, 1)
    assert p.fetch_frames.tolist() == [0, 1]
    o.pool_words[0, 3] = 111
    o.pool_words[1, 5] = 222
    p = o.plan([(0, 1)]); o.migrate(); o.launch_retire(0, 1)
    assert p.evict_pages.tolist() == [0, 1] and p.fetch_pages.tolist() == [2, 3]
    assert o.host_words[0, 3] == 111 and o.host_words[1, 5] == 222
    assert np.array_equal(o.pool_words, page_words([2, 3], wpp))
    p = o.plan([(0, 1)]); o.migrate()
    assert o.pool_words[0, 3] == 111 and o.pool_words[1, 5] == 222
    assert o.pagetable_query([0, 1, 2, 3]).tolist() == [0, 1, NONE, NONE]


def test_lru_textbook_cases(oracle_mod):
    # pool >= footprint: compulsory misses only
    cmds = [[[0, 1], [2], [0, 3], [1, 2]], [[4], [5, 0], [4]]]
    trace = explicit_trace(cmds, 8, 8, timeslice=1)
    o = oracle_mod.Oracle.for_trace(trace)
    load_trace(o, trace)
    order = [(0, 0), (1, 0), (0, 1), (1, 1), (0, 2), (1, 2), (0, 3)]
    t, i = zip(*order)
    assert o.lru_faults(t, i, 8) == 6
    # cyclic sweep over one more page than fits: every reference misses
    sweep = [[[p] for p in range(5)] * 4]
    trace = explicit_trace(sweep, 5, 4, timeslice=1)
    o = oracle_mod.Oracle.for_trace(trace)
    load_trace(o, trace)
    assert o.lru_faults([0] * 20, list(range(20)), 4) == 20
    # a hand-worked string, capacity 3: 1 2 3 1 4 2 5 1 -> misses at 1 2 3 . 4(ev 2) 2(ev 3) 5(ev 1) 1(ev 4)
    s = [1, 2, 3, 1, 4, 2, 5, 1]
    trace = explicit_trace([[[p] for p in s]], 8, 3, timeslice=1)
    o = oracle_mod.Oracle.for_trace(trace)
    load_trace(o, trace)
    assert o.lru_faults([0] * len(s), list(range(len(s))), 3) == 7
