"""HIP path vs CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import sys

import numpy as np
import pytest

from workloads import make_trace, Rule, RULE_LIST, RULE_LINEAR
from helpers import explicit_trace
from gpu_common import lockstep, GpuSide, make_oracle, assert_same_plan

pytestmark = pytest.mark.gpu


def _log(msg):
    print(msg, flush=True)


def test_c1_tiny_round_robin_full_size(oracle_mod):
    for seed in (0, 1):
        n = lockstep(oracle_mod, make_trace(1, seed=seed), with_bytes=True)
        assert n >= 20


def test_c2_stencil_page_structure_small_pages(oracle_mod):
    assert lockstep(oracle_mod, make_trace(2, page_shift=14), with_bytes=True, bytes_every=8) == 80


def test_c3_training_scaled_with_cut_slices(oracle_mod):
    trace = make_trace(3, page_shift=12, scale=32, layers=8, iterations=3)
    n = lockstep(oracle_mod, trace, with_bytes=True, bytes_every=4, log=_log)
    assert n >= 6


def test_c4_decode_scaled_strided_rules_sparse_slots(oracle_mod):
    trace = make_trace(4, page_shift=12, layers=8, steps=24)
    assert lockstep(oracle_mod, trace, with_bytes=True, bytes_every=3) >= 12


def test_c5_planning_stress_scaled(oracle_mod):
    trace = make_trace(5, scale=64, n_launches=100)
    assert lockstep(oracle_mod, trace, with_bytes=True, bytes_every=4, log=_log) >= 16


def test_full_horizon_timelines_tiny_random(oracle_mod):
    rng = np.random.default_rng(21)
    for trial in range(25):
        n_tasks = int(rng.integers(1, 4))
        n_pages = int(rng.integers(5, 70))
        n_frames = int(rng.integers(4, 9))
        cmds = [[sorted(rng.choice(n_pages, size=int(rng.integers(1, 4)), replace=False).tolist())
                 for _ in range(int(rng.integers(2, 9)))] for _ in range(n_tasks)]
        trace = explicit_trace(cmds, n_pages, n_frames, int(rng.integers(1, 4)), page_shift=6)
        lockstep(oracle_mod, trace, with_bytes=True, horizon="full")


def test_many_commands_in_one_timeline(oracle_mod):
    # G in the thousands: one task, 3000 one-page launches, full horizon
    rng = np.random.default_rng(2)
    cmds = [[[int(rng.integers(0, 500))] for _ in range(3000)]]
    trace = explicit_trace(cmds, 500, 64, timeslice=100, page_shift=6)
    assert lockstep(oracle_mod, trace, with_bytes=True, horizon="full", max_plans=4) == 4


def test_next_use_epoch_wraps_cleanly(oracle_mod, monkeypatch):
    # the next-use array is never cleared between plans: entries carry a plan epoch that wraps
    # after 2^20 - 1 plans; start 5 plans before the wrap and run across it
    monkeypatch.setenv("MSCHED_INITIAL_EPOCH", str((1 << 20) - 6))
    assert lockstep(oracle_mod, make_trace(1, seed=4), with_bytes=True) >= 20


def test_errors_and_edge_cases(oracle_mod):
    from paper_2512_24637_amd import MSchedError
    trace = explicit_trace([[[0, 1, 2, 3], [4]], [[5]]], 8, 3, timeslice=1, page_shift=6)
    g = GpuSide(trace)
    try:
        ms = g.ms
        with pytest.raises(MSchedError) as e:           # first command alone exceeds the pool
            ms.plan([(0, 1)])
        assert e.value.name == "E_WSET_TOO_LARGE"
        p = ms.plan([])                                 # empty timeline plans nothing
        assert (p.n_fetch, p.n_evict, p.covered_launches) == (0, 0, 0)
        ms.migrate(p)
        with pytest.raises(MSchedError) as e:           # a plan can be carried out once
            ms.migrate(p)
        assert e.value.name == "E_STALE_PLAN"
        p1 = ms.plan([(1, 1)])
        p2 = ms.plan([(1, 1)])
        with pytest.raises(MSchedError) as e:           # only the latest plan may be carried out
            ms.migrate(p1)
        assert e.value.name == "E_STALE_PLAN"
        ms.migrate(p2)
        assert ms.pagetable_query([5, 0]).tolist() == [0, 0xFFFFFFFF]
        with pytest.raises(MSchedError) as e:
            ms.pagetable_query([8])
        assert e.value.name == "E_RANGE"
        with pytest.raises(MSchedError) as e:           # unknown task in the timeline
            ms.plan([(7, 1)])
        assert e.value.name == "E_INVAL"
        k = ms.kernel_register([Rule(RULE_LINEAR, 0, (1, 2), 1 << 40)])
        with pytest.raises(MSchedError) as e:
            ms.launch_enqueue(1, k, [0, 1 << 20, 1 << 20], 3)
        assert e.value.name == "E_OVERFLOW"
        with pytest.raises(MSchedError) as e:
            ms.launch_enqueue(1, k, [0, 1], 2)
        assert e.value.name == "E_RANGE"
        k2 = ms.kernel_register([Rule(RULE_LINEAR, 0, (1,), 1)])
        with pytest.raises(MSchedError) as e:
            ms.launch_enqueue(1, k2, [7 * 64, 65], 2)
        assert e.value.name == "E_RANGE"
        with pytest.raises(MSchedError) as e:
            ms.launch_enqueue(1, k2, [(1 << 64) - 10, 100], 2)
        assert e.value.name == "E_OVERFLOW"
        # a LIST id beyond the page table is caught while planning; state is untouched
        import torch
        bad = torch.tensor([1, 2, 99], dtype=torch.int32, device="cuda")
        kl = ms.kernel_register([Rule(RULE_LIST)])
        ms.launch_retire(1, 1)
        ms.launch_enqueue(1, kl, [], 0, ids_ptr=bad.data_ptr(), n_ids=3)
        before = ms.state()
        with pytest.raises(MSchedError) as e:
            ms.plan([(1, 1)])
        assert e.value.name == "E_RANGE"
        after = ms.state()
        assert np.array_equal(before[0], after[0]) and np.array_equal(before[1], after[1])
    finally:
        g.close()
