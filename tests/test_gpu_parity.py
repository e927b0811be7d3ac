"""HIP path vs CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import sys

import numpy as np
import pytest

from workloads import make_trace, run_schedule, Rule, RULE_LIST, RULE_LINEAR
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


@pytest.mark.parametrize("n_pages,force_multi", [(500, True), (20000, False)])
def test_many_commands_through_the_multi_kernel_cut(oracle_mod, monkeypatch, n_pages, force_multi):
    """G = 3000 classes through the stand-alone cut (few chunks) and through the cut fused with the column
    prefixes (79 chunks): a wavefront's scan then walks 47 classes per lane."""
    if force_multi:
        monkeypatch.setenv("MSCHED_FORCE_MULTI_KERNEL", "1")
    rng = np.random.default_rng(12)
    cmds = [[[int(rng.integers(0, n_pages))] for _ in range(3000)]]
    trace = explicit_trace(cmds, n_pages, 64, timeslice=100, page_shift=6)
    assert lockstep(oracle_mod, trace, with_bytes=True, horizon="full", max_plans=3) == 3


@pytest.mark.parametrize("n_ranges", [16, 31, 32, 33, 34, 63, 64, 65, 66, 70, 118])
@pytest.mark.parametrize("force_multi", [False, True])
def test_ranges_per_tile_around_the_limit_of_the_register_path(oracle_mod, monkeypatch, n_ranges, force_multi):
    """Up to 32 partial ranges of a tile are applied from registers, more are painted in LDS (short ones by the thread
    that finds them, longer ones through a queue of 64, then in place): n short ranges inside one tile, long ranges
    that cover whole tiles and end inside others, and the table's ragged end; the second plan has to evict part of
    what the first brought in."""
    if force_multi:
        monkeypatch.setenv("MSCHED_FORCE_MULTI_KERNEL", "1")
    V, F, P = 6000, 3000, 64
    trace = explicit_trace([[[0]], [[1]]], V, F, timeslice=4, page_shift=6)
    g = GpuSide(trace)
    o = make_oracle(oracle_mod, trace, with_bytes=False)
    rng = np.random.default_rng(n_ranges)
    try:
        rule = [Rule(RULE_LINEAR, 0, (1,), P)]
        kg, ko = g.ms.kernel_register(rule), o.kernel_register(rule)
        for impl in (g.ms, o):
            impl.launch_retire(0, 1)
            impl.launch_retire(1, 1)
        starts = rng.permutation(120)[:n_ranges - 1] * 4 + 20            # short ranges, 3 pages each, inside pages [20, 500)
        cmds0 = [(int(a), 3) for a in starts] + [(2500, 1500)]           # and one long range further up
        cmds1 = [(0, 2800), (4000, 100), (5990, 10)]                     # whole tiles and the short ranges' pages; elsewhere; the ragged end
        for task, cmds, k in ((0, cmds0, (kg, ko)), (1, cmds1, (kg, ko))):
            for a, n in cmds:
                g.ms.launch_enqueue(task, k[0], [a * P, n], 2)
                o.launch_enqueue(task, k[1], [a * P, n], 2)
        for tl in ([(0, len(cmds0)), (1, 3)], [(1, 3), (0, len(cmds0))], [(0, 7), (1, 1)]):
            po, pg = o.plan(tl), g.ms.plan(tl)
            assert_same_plan(po, pg, tl)
            o.migrate()
            g.ms.migrate()
            pto, foo = o.state()
            ptg, fog = g.ms.state()
            assert np.array_equal(pto, ptg) and np.array_equal(foo, fog)
    finally:
        g.close()
        o.close()


def test_a_chunk_remembers_for_some_plans_that_its_ranges_overflowed(oracle_mod, monkeypatch):
    """A chunk whose tile met more partial ranges than are applied from registers paints the next 16 plans' ranges in
    LDS without trying the queue; then it tries the queue again.  Timelines with 70 short ranges in one tile and
    with 3 alternate over 45 plans, so that every combination is passed through: overflow with and without the
    hint set, few ranges with the hint set (painted in LDS), and after it has run out (applied from registers)."""
    monkeypatch.setenv("MSCHED_FORCE_MULTI_KERNEL", "1")
    V, F, P = 6000, 3000, 64
    trace = explicit_trace([[[0]], [[1]]], V, F, timeslice=4, page_shift=6)
    g = GpuSide(trace)
    o = make_oracle(oracle_mod, trace, with_bytes=False)
    rng = np.random.default_rng(5)
    try:
        rule = [Rule(RULE_LINEAR, 0, (1,), P)]
        kg, ko = g.ms.kernel_register(rule), o.kernel_register(rule)
        for impl in (g.ms, o):
            impl.launch_retire(0, 1)
            impl.launch_retire(1, 1)
        starts = rng.permutation(120)[:69] * 4 + 20
        cmds0 = [(int(a), 3) for a in starts] + [(2500, 1500)]
        cmds1 = [(0, 2800), (4000, 100), (5990, 10)]
        for task, cmds in ((0, cmds0), (1, cmds1)):
            for a, n in cmds:
                g.ms.launch_enqueue(task, kg, [a * P, n], 2)
                o.launch_enqueue(task, ko, [a * P, n], 2)
        many, few = [(0, len(cmds0)), (1, 3)], [(1, 3), (0, 5)]
        for i in range(45):
            tl = many if i in (0, 1, 5, 30, 31) else few
            po, pg = o.plan(tl), g.ms.plan(tl)
            assert_same_plan(po, pg, tl)
            o.migrate()
            g.ms.migrate()
            pto, foo = o.state()
            ptg, fog = g.ms.state()
            assert np.array_equal(pto, ptg) and np.array_equal(foo, fog), i
    finally:
        g.close()
        o.close()


def test_next_use_epoch_wraps_cleanly(oracle_mod, monkeypatch):
    # the next-use array is never cleared between plans: entries carry a plan epoch that wraps
    # after 2^20 - 1 plans; start 5 plans before the wrap and run across it
    monkeypatch.setenv("MSCHED_INITIAL_EPOCH", str((1 << 20) - 6))
    assert lockstep(oracle_mod, make_trace(1, seed=4), with_bytes=True) >= 20


def test_small_tables_also_pass_through_the_multi_kernel_path(oracle_mod, monkeypatch):
    # page tables of up to 8 Ki pages normally take the fused single-workgroup kernel
    monkeypatch.setenv("MSCHED_FORCE_MULTI_KERNEL", "1")
    assert lockstep(oracle_mod, make_trace(1, seed=2), with_bytes=True) >= 20
    assert lockstep(oracle_mod, make_trace(4, page_shift=12, layers=8, steps=16), with_bytes=True, bytes_every=3) >= 8


def test_id_lists_through_the_bucket_path(oracle_mod, monkeypatch):
    # plans with many ids bin them by page bucket instead of scattering atomics; force it for small lists
    monkeypatch.setenv("MSCHED_LIST_BINNED_MIN_IDS", "0")
    trace = make_trace(5, scale=64, n_launches=100)
    assert lockstep(oracle_mod, trace, with_bytes=True, bytes_every=4) >= 16
    rng = np.random.default_rng(77)
    trace = _random_rule_trace(rng, page_shift=8, V=70000, n_frames=9000, n_tasks=3, n_cmds=24, with_lists=True)
    assert lockstep(oracle_mod, trace, with_bytes=True, bytes_every=6) >= 8


def test_launches_arriving_between_switches(oracle_mod):
    # launches are enqueued only two or three timeslices ahead, so queues grow while their heads retire
    assert lockstep(oracle_mod, make_trace(1, seed=6, n_launches=900), with_bytes=True, bytes_every=7,
                    lazy_slices=2) >= 90
    assert lockstep(oracle_mod, make_trace(4, page_shift=12, layers=8, steps=40), with_bytes=True, bytes_every=5,
                    lazy_slices=3) >= 20
    # a queue in steady state: 800 launches pass through a record array of 256, which is compacted in place
    assert lockstep(oracle_mod, make_trace(1, seed=9, n_launches=2400), with_bytes=True, bytes_every=40,
                    lazy_slices=1) >= 240


@pytest.mark.parametrize("binned", [False, True])
def test_list_id_without_backing_slot_is_refused_at_plan_time(oracle_mod, monkeypatch, binned):
    import torch
    from paper_2512_24637_amd import MSchedError
    if binned:
        monkeypatch.setenv("MSCHED_LIST_BINNED_MIN_IDS", "0")
    trace = explicit_trace([[[0, 1]]], 64, 8, timeslice=1, page_shift=6)
    slot = np.full(64, 0xFFFFFFFF, np.uint32)
    slot[:32] = np.arange(32)                            # pages 32..63 have no backing store
    trace.host_slot, trace.n_slots = slot, 32
    g = GpuSide(trace)
    try:
        ms = g.ms
        kl = ms.kernel_register([Rule(RULE_LIST)])
        ok = torch.tensor([3, 5, 3, 31], dtype=torch.int32, device="cuda")
        bad = torch.tensor([3, 40, 5], dtype=torch.int32, device="cuda")
        ms.launch_retire(0, 1)
        ms.launch_enqueue(0, kl, [], 0, ids_ptr=ok.data_ptr(), n_ids=4)
        p = ms.plan([(0, 1)])
        assert p.fetch_pages.tolist() == [3, 5, 31]
        ms.migrate(p)
        ms.launch_retire(0, 1)
        ms.launch_enqueue(0, kl, [], 0, ids_ptr=bad.data_ptr(), n_ids=3)
        with pytest.raises(MSchedError) as e:
            ms.plan([(0, 1)])
        assert e.value.name == "E_RANGE"
        assert ms.pagetable_query([3, 5, 31, 40]).tolist() == [0, 1, 2, 0xFFFFFFFF]
    finally:
        g.close()


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


def _random_rule_trace(rng, page_shift, V, n_frames, n_tasks, n_cmds, with_lists):
    """Random templates of every kind (fixed, linear in 1-3 arguments, strided with small, large,
    abutting and overlapping chunks, id lists with repeats) and random launches that stay in range."""
    from workloads import Trace, RULE_FIXED, RULE_STRIDED
    from workloads.trace import CommandBuilder
    P = 1 << page_shift
    n_bytes = V * P
    kernels, makers = [], []
    for k in range(12):
        n_rules = int(rng.integers(1, 5))
        rules, parts = [], []
        n_args = 0
        for r in range(n_rules):
            kind = int(rng.choice([RULE_FIXED, RULE_LINEAR, RULE_STRIDED] + ([RULE_LIST] if with_lists and r == 0 else [])))
            if kind == RULE_LIST:
                rules.append(Rule(RULE_LIST)); parts.append(("list",)); continue
            if n_args > 8:
                break
            base_idx = n_args; n_args += 1
            if kind == RULE_FIXED:
                size = int(rng.integers(0, 40 * P))
                rules.append(Rule(RULE_FIXED, base_idx, (), size)); parts.append(("fixed", size))
            elif kind == RULE_LINEAR:
                m = int(rng.integers(1, 3))
                idx = tuple(range(n_args, n_args + m)); n_args += m
                coeff = int(rng.choice([1, 2, 4, 8]))
                rules.append(Rule(RULE_LINEAR, base_idx, idx, coeff)); parts.append(("linear", m, coeff))
            else:
                idx = (n_args, n_args + 1, n_args + 2); n_args += 3
                cs, cst = int(rng.choice([1, 16, 64])), int(rng.choice([1, 16, 64]))
                rules.append(Rule(RULE_STRIDED, base_idx, (idx[0],), cs, (idx[1],), cst, (idx[2],), 1))
                parts.append(("strided", cs, cst))
        kernels.append(rules); makers.append((parts, n_args))
    tasks, pools, off = [], [], 0
    for t in range(n_tasks):
        b = CommandBuilder()
        for _ in range(n_cmds):
            k = int(rng.integers(0, len(kernels)))
            parts, n_args = makers[k]
            args, n_ids, ids_off = [], 0, 0
            for part in parts:
                if part[0] == "list":
                    n_ids = int(rng.integers(0, 200))
                    pools.append(rng.integers(0, V, size=n_ids).astype(np.uint32)); ids_off = off; off += n_ids
                    continue
                span_cap = min(n_bytes // 2, 60 * P)
                if part[0] == "fixed":
                    args.append(int(rng.integers(0, n_bytes - part[1] + 1)))
                elif part[0] == "linear":
                    vals = [int(rng.integers(0, 40)) for _ in range(part[1])]
                    size = part[2] * int(np.prod(vals))
                    while size > span_cap:
                        vals[0] = max(0, vals[0] // 2); size = part[2] * int(np.prod(vals))
                    args.append(int(rng.integers(0, n_bytes - size + 1))); args.extend(vals)
                else:
                    chunk_n = int(rng.integers(0, 30 * P // part[1] + 1))       # up to ~30 pages per chunk
                    stride_n = int(rng.integers(0, 40 * P // part[2] + 1))
                    count = int(rng.integers(0, 6))
                    span = (max(count, 1) - 1) * stride_n * part[2] + chunk_n * part[1]
                    while span > n_bytes // 2:
                        stride_n //= 2; chunk_n //= 2
                        span = (max(count, 1) - 1) * stride_n * part[2] + chunk_n * part[1]
                    args.append(int(rng.integers(0, n_bytes - span + 1))); args.extend([chunk_n, stride_n, count])
            b.add(k, args, latency=int(rng.integers(1, 4)), ids_off=ids_off, n_ids=n_ids)
        tasks.append(b.build())
    ids_pool = np.concatenate(pools).astype(np.uint32) if pools else np.zeros(0, np.uint32)
    return Trace(name="random-rules", page_shift=page_shift, n_virtual_pages=V, n_frames=n_frames,
                 timeslice=4, kernels=kernels, tasks=tasks, ids_pool=ids_pool, n_slots=V)


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4, 5])
def test_random_templates_of_every_kind(oracle_mod, seed):
    rng = np.random.default_rng(100 + seed)
    V = int(rng.choice([700, 3000, 9000])) if seed < 4 else {4: 20000, 5: 70000}[seed]   # 5: many chunks, fused cut
    trace = _random_rule_trace(rng, page_shift=8, V=V, n_frames=V // 3 + 200, n_tasks=3, n_cmds=30,
                               with_lists=bool(seed % 2))
    assert lockstep(oracle_mod, trace, with_bytes=True, bytes_every=5) >= 10


@pytest.mark.parametrize("announce", [False, True])
def test_priority_policy_with_profiled_latencies(oracle_mod, announce):
    """Real-time inference preempting best-effort training: latency-weighted slices, a timeline that changes
    shape between switches, requests enqueued while the schedule runs."""
    from workloads import run_priority_schedule
    trace = make_trace(6, scale=16)
    driver = lambda tr, impl, max_plans: run_priority_schedule(tr, impl, max_plans, announce_next_request=announce)
    assert lockstep(oracle_mod, trace, with_bytes=True, bytes_every=3, driver=driver) >= 15


def test_allocation_granularity_ablation_runs_bit_exact(oracle_mod):
    """The naive predictor's schedule (whole buffers per pointer) through the same path: larger working sets,
    slices cut to what fits, replans inside a timeslice."""
    from workloads.ablation import allocation_granularity
    trace = allocation_granularity(make_trace(4, page_shift=15, steps=12, full_backing=True))
    assert lockstep(oracle_mod, trace, with_bytes=True, bytes_every=4) >= 20


@pytest.mark.parametrize("env", [{"MSCHED_PAINT": "0"}, {"MSCHED_LIST_PREPARED": "0"},
                                 {"MSCHED_PAINT": "0", "MSCHED_LIST_PREPARED": "0"},
                                 {"MSCHED_LIST_CACHE_MB": "1"}, {"MSCHED_LIST_AHEAD": "0"}, {"MSCHED_PLAN_SPIN": "0"},
                                 {"MSCHED_MAX_CHUNKS": "16"}, {"MSCHED_MAX_CHUNKS": "16", "MSCHED_FUSE_LISTS": "0"},
                                 {"MSCHED_MAX_CHUNKS": "16", "MSCHED_LIST_AHEAD": "0"}, {"MSCHED_ORDER_EMIT": "0"}],
                         ids=["scatter-ranges", "bin-per-plan", "both-earlier-paths", "one-megabyte-ring", "no-look-ahead",
                              "plan-waits-for-the-stream", "lists-merged-in-the-sweep", "full-size-tiles-own-merge",
                              "lists-merged-in-the-sweep-no-look-ahead", "second-sweep-in-strided-order"])
def test_earlier_planning_paths_stay_bit_exact(oracle_mod, monkeypatch, env):
    """Range pages scattered into the next-use array instead of painted, id lists binned from scratch in every
    plan instead of prepared once per command, a ring too small for the prepared lists (which makes plans fall
    back to binning from scratch part of the time), lists prepared by the plan that first sees them instead of
    behind the previous migration, and a plan call that waits for the whole stream instead of the stamped counts.
    With at most 16 sweep workgroups the scaled tables get the full-size tiles (one bucket of id lists each) of
    the large ones, where the first sweep merges the prepared lists itself - or, switched off, leaves that to the
    merge kernel.  Last, the second sweep taking its chunks in the strided order of the first instead of those
    that may list pages first."""
    monkeypatch.setenv("MSCHED_LIST_BINNED_MIN_IDS", "0")
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    assert lockstep(oracle_mod, make_trace(5, scale=64, n_launches=100), with_bytes=True, bytes_every=4) >= 16
    assert lockstep(oracle_mod, make_trace(3, scale=16, iterations=2), with_bytes=True, bytes_every=3) >= 4
    assert lockstep(oracle_mod, make_trace(4, page_shift=12, layers=8, steps=16), with_bytes=True, bytes_every=3) >= 8


@pytest.mark.parametrize("case", ["one-launch-of-5000-chunks", "6000-chunks-over-300-launches"])
def test_more_ranges_than_the_range_list_holds(oracle_mod, case):
    """Plans whose range rules do not fit the list the sweeps paint from (4096 ranges) scatter next uses per page
    instead: a single launch whose strided rule has 5000 one-page chunks (nothing is kept of its ranges when it is
    queued), and 300 launches of 20 chunks each (every launch fits, the plan does not).  Launches that repeat a region
    of a queued launch, and plain ranges beside the strided ones, go through the same plans."""
    from workloads import Trace, RULE_STRIDED
    from workloads.trace import CommandBuilder
    P = 64
    strided = [Rule(RULE_STRIDED, 0, (1,), 1, (2,), 1, (3,), 1)]          # args: base, chunk bytes, stride bytes, chunks
    linear = [Rule(RULE_LINEAR, 0, (1,), 1)]
    both = [Rule(RULE_STRIDED, 0, (2,), 1, (3,), 1, (4,), 1), Rule(RULE_LINEAR, 1, (5,), 1)]
    kernels = [strided, linear, both]
    t0, t1 = CommandBuilder(), CommandBuilder()
    if case == "one-launch-of-5000-chunks":
        V, F, slice_len = 40000, 9000, 3
        for rep in range(4):
            t0.add(0, [0, P, 2 * P, 5000])                                  # pages 0, 2, ..., 9998
            t0.add(1, [12000 * P + 8, 500 * P])                             # a ragged plain range
            t0.add(0, [0, P, 2 * P, 5000])                                  # the same region again
            t0.add(2, [20000 * P, 30000 * P, 3 * P, 7 * P, 40, 100 * P])    # 40 chunks of 3 pages + a plain range
            t1.add(0, [1 * P, P, 2 * P, 4500])                              # the odd pages
            t1.add(1, [35000 * P, 2000 * P])
            t1.add(2, [20000 * P, 30000 * P, 3 * P, 7 * P, 40, 100 * P])    # task 0's region, from another task
    else:
        V, F, slice_len = 40000, 12000, 150
        rng = np.random.default_rng(5)
        for t in (t0, t1):
            for i in range(300):
                base = int(rng.integers(0, 30000))
                t.add(0, [base * P, 2 * P, 9 * P, 20])                      # 20 chunks of 2 pages
                if i % 7 == 0:
                    t.add(0, [base * P, 2 * P, 9 * P, 20])                  # a repeat right behind it
    trace = Trace(name=case, page_shift=6, n_virtual_pages=V, n_frames=F, timeslice=slice_len, kernels=kernels,
                  tasks=[t0.build(), t1.build()], n_slots=V)
    assert lockstep(oracle_mod, trace, with_bytes=True, bytes_every=2) >= 4


@pytest.mark.parametrize("early", [False, True], ids=["plain", "early-execution"])
def test_pages_larger_than_a_work_unit_of_the_copy(oracle_mod, monkeypatch, early):
    """Pages of several chunks: 4 MiB pages (two 2 MiB chunks each; 64 chunks of 64 KiB under early execution) on
    the tiny round-robin schedule, then its 64 KiB pages cut into 16 chunks of 4 KiB by the launch-shape hook.
    The page is mapped by the workgroup that finishes its last chunk; plans, tables and every byte must equal the
    oracle's after every switch."""
    from workloads.harness import load_trace
    for page_shift, chunk in ((22, None), (16, "12")):
        if chunk:
            monkeypatch.setenv("MSCHED_MIGRATE_CHUNK_SHIFT", chunk)
            monkeypatch.setenv("MSCHED_EARLY_CHUNK_SHIFT", chunk)
        trace = make_trace(1, seed=3, page_shift=page_shift, n_launches=60)     # 384 pages, 256 frames: 1 GiB pool at 4 MiB
        if not early:
            assert lockstep(oracle_mod, trace, with_bytes=True, bytes_every=2) >= 6
            continue
        g = GpuSide(trace)
        o = make_oracle(oracle_mod, trace, with_bytes=True)
        try:
            g.ms.set_early_start(True)
            n = 0
            for ro, rg in zip(run_schedule(trace, o), run_schedule(trace, g.ms)):
                assert_same_plan(ro.plan, rg.plan, (trace.name, ro.index))
                assert g.ms.progress() <= rg.plan.n_fetch
                pto, foo = o.state()
                ptg, fog = g.ms.state()
                assert np.array_equal(pto, ptg) and np.array_equal(foo, fog)
                assert g.ms.progress() == rg.plan.n_fetch          # the stream has drained: everything has landed
                if n % 2 == 0:
                    assert np.array_equal(o.pool_words, g.pool_words())
                    assert np.array_equal(o.host_words, g.host_words())
                n += 1
            assert n >= 6
        finally:
            g.close()
            o.close()


@pytest.mark.parametrize("env", [{}, {"MSCHED_FUSE_LISTS": "0"}, {"MSCHED_LIST_AHEAD": "0"}], ids=["merged-in-the-sweep", "own-merge-kernel", "no-look-ahead"])
def test_id_lists_prepared_in_parts_by_bucket_range(oracle_mod, monkeypatch, env):
    """With MSCHED_PREP_SPLIT every piece of an id list of a table of 32 buckets or more is prepared by several
    workgroups, part q taking the buckets q, q + parts, ...: 80 buckets in 4 parts here (config 5 at 1/16 of its
    pages, 64-byte pages), 40 buckets in 2 parts at 1/32."""
    monkeypatch.setenv("MSCHED_LIST_BINNED_MIN_IDS", "0")
    monkeypatch.setenv("MSCHED_PREP_SPLIT", "4")
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    for scale in (16, 32):
        trace = make_trace(5, scale=scale, page_shift=6, n_launches=100)
        assert lockstep(oracle_mod, trace, with_bytes=True, bytes_every=5) >= 16


@pytest.mark.parametrize("env", [{}, {"MSCHED_DEDUPE_REGIONS": "0"}, {"MSCHED_RESIDENT_RANGES": "0"}],
                         ids=["ranges-through-mirrors", "mirrors-no-repeats-dropped", "ranges-listed-per-plan"])
def test_ranges_through_the_tasks_mirrors(oracle_mod, monkeypatch, env):
    """Sweeps of large tables whose plans carry no id lists read the page ranges through per-task mirrors in device
    memory, a wavefront serving one run of the timeline, instead of through a list made and copied per plan: the
    DL-training and decode schedules at page sizes that give them multi-workgroup sweeps, launches arriving as they
    go; plans with id lists (config 5 at 1/8 and 1/16 of its pages) keep their staged tables.  The last case lists
    and copies the ranges per plan as before."""
    monkeypatch.setenv("MSCHED_LIST_BINNED_MIN_IDS", "0")
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    for scale, lazy in ((8, None), (16, 2)):
        trace = make_trace(5, scale=scale, page_shift=6, n_launches=100)
        assert lockstep(oracle_mod, trace, with_bytes=True, bytes_every=5, lazy_slices=lazy) >= 16
    assert lockstep(oracle_mod, make_trace(3, page_shift=12, scale=32, layers=8, iterations=3), with_bytes=True, bytes_every=3) >= 4
    assert lockstep(oracle_mod, make_trace(3, page_shift=12, scale=32, layers=8, iterations=4), with_bytes=False, lazy_slices=1) >= 6
    assert lockstep(oracle_mod, make_trace(4, page_shift=12, layers=8, steps=24), with_bytes=True, bytes_every=5, lazy_slices=2) >= 10


def test_id_lists_longer_than_one_prepared_piece(oracle_mod, monkeypatch):
    """A list of 60 000 ids is prepared as three pieces of up to 24 576; the same list object repeated by a later
    command is skipped, a different list over the same pages is merged."""
    import torch
    monkeypatch.setenv("MSCHED_LIST_BINNED_MIN_IDS", "0")
    V, F = 40000, 38000
    trace = explicit_trace([[[0]], [[1]]], V, F, timeslice=4, page_shift=6)
    g = GpuSide(trace)
    o = make_oracle(oracle_mod, trace, with_bytes=False)
    rng = np.random.default_rng(3)
    try:
        lists = [rng.integers(0, V, 60000).astype(np.uint32), rng.integers(0, V // 2, 30000).astype(np.uint32),
                 rng.integers(V // 3, V, 5).astype(np.uint32)]
        dev = [torch.from_numpy(a.view(np.int32)).cuda() for a in lists]
        kg = g.ms.kernel_register([Rule(RULE_LIST)])
        ko = o.kernel_register([Rule(RULE_LIST)])
        for impl, k in ((g.ms, kg), (o, ko)):
            impl.launch_retire(0, 1)
            impl.launch_retire(1, 1)
        for task, which in ((0, 1), (0, 0), (1, 2), (0, 0), (1, 1)):
            g.ms.launch_enqueue(task, kg, [], 0, ids_ptr=dev[which].data_ptr(), n_ids=len(lists[which]))
            o.launch_enqueue(task, ko, [], 0, ids=lists[which])
        for tl, retire in (([(0, 1), (1, 4)], (0, 1)), ([(1, 1), (0, 4)], (1, 1)), ([(0, 2), (1, 4)], (0, 2)), ([(1, 4)], (1, 1))):
            po, pg = o.plan(tl), g.ms.plan(tl)
            assert_same_plan(po, pg, tl)
            o.migrate()
            g.ms.migrate()
            pto, foo = o.state()
            ptg, fog = g.ms.state()
            assert np.array_equal(pto, ptg) and np.array_equal(foo, fog)
            o.launch_retire(*retire)
            g.ms.launch_retire(*retire)
    finally:
        g.close()
        o.close()


def test_a_plan_with_more_than_a_thousand_prepared_lists(oracle_mod, monkeypatch):
    """1300 commands, each with a short id list of its own: the merge keeps a table entry per list in LDS, which
    at this count asks for more than 64 KiB per workgroup."""
    import torch
    monkeypatch.setenv("MSCHED_LIST_BINNED_MIN_IDS", "0")
    V, F, n_cmds, n_ids = 40000, 30000, 650, 48
    trace = explicit_trace([[[0]], [[1]]], V, F, timeslice=n_cmds, page_shift=6)
    g = GpuSide(trace)
    o = make_oracle(oracle_mod, trace, with_bytes=False)
    rng = np.random.default_rng(17)
    try:
        ids = rng.integers(0, V, (2, n_cmds, n_ids)).astype(np.uint32)
        dev = torch.from_numpy(ids.view(np.int32)).cuda()
        kg = g.ms.kernel_register([Rule(RULE_LIST)])
        ko = o.kernel_register([Rule(RULE_LIST)])
        for impl in (g.ms, o):
            impl.launch_retire(0, 1)
            impl.launch_retire(1, 1)
        for task in (0, 1):
            for i in range(n_cmds):
                g.ms.launch_enqueue(task, kg, [], 0, ids_ptr=dev[task, i].data_ptr(), n_ids=n_ids)
                o.launch_enqueue(task, ko, [], 0, ids=ids[task, i])
        for k, tl in enumerate(([(0, n_cmds), (1, n_cmds)], [(1, n_cmds), (0, n_cmds)], [(0, n_cmds), (1, n_cmds)])):
            po, pg = o.plan(tl), g.ms.plan(tl)
            if k == 0:
                assert pg.n_commands == 2 * n_cmds
            assert_same_plan(po, pg, tl)
            o.migrate()
            g.ms.migrate()
            pto, foo = o.state()
            ptg, fog = g.ms.state()
            assert np.array_equal(pto, ptg) and np.array_equal(foo, fog)
            n = min(po.covered_launches, 200)                  # the rest of the slice stays queued: most lists are planned again
            o.launch_retire(tl[0][0], n)
            g.ms.launch_retire(tl[0][0], n)
    finally:
        g.close()
        o.close()


@pytest.mark.parametrize("layout", ["everywhere", "apart"])
def test_lists_merged_in_the_sweep_more_pieces_than_one_staging_round(oracle_mod, monkeypatch, layout):
    """Full-size tiles (three sweep workgroups for 70 000 pages, the last tile ragged) and 402 commands whose lists
    of 60 000 ids are prepared as three pieces each: the sweep describes a bucket's 1206 segments in LDS in two
    rounds.  Then a list with an id beyond the table, which the sweep of bucket 0 has to report.
    "everywhere": every tile holds ids and dozens of short ranges (painted in LDS, lists merged on top).
    "apart": the ids stay in the upper half of the table; most commands repeat one range (described once per
    plan), a few bring long ranges of their own in the lower half, so the tiles there hold no ids and only a few
    ranges (applied from registers), and one range reaches into the tiles with ids."""
    import torch
    from paper_2512_24637_amd import MSchedError
    monkeypatch.setenv("MSCHED_LIST_BINNED_MIN_IDS", "0")
    monkeypatch.setenv("MSCHED_MAX_CHUNKS", "3")
    V, F, n_cmds, n_ids = 70000, 50000, 201, 60000
    trace = explicit_trace([[[0]], [[1]]], V, F, timeslice=n_cmds, page_shift=6)
    g = GpuSide(trace)
    o = make_oracle(oracle_mod, trace, with_bytes=False)
    rng = np.random.default_rng(23)
    try:
        # every command reads one window of a quarter of the table; the windows move with the command
        lo = rng.integers(V // 2 if layout == "apart" else 0, V - V // 4, (2, n_cmds))
        ids = (lo[:, :, None] + rng.integers(0, V // 4, (2, n_cmds, n_ids))).astype(np.uint32)
        dev = torch.from_numpy(ids.view(np.int32)).cuda()
        kg = g.ms.kernel_register([Rule(RULE_LINEAR, 0, (1,), 4), Rule(RULE_LIST)])
        ko = o.kernel_register([Rule(RULE_LINEAR, 0, (1,), 4), Rule(RULE_LIST)])
        for impl in (g.ms, o):
            impl.launch_retire(0, 1)
            impl.launch_retire(1, 1)
        for task in (0, 1):
            for i in range(n_cmds):
                args = [int(rng.integers(0, V - 600)) * 64, int(rng.integers(1, 500)) * 16]
                if layout == "apart":
                    args = [1000 * 64, 300 * 16]
                    if i % 40 == 7:
                        args = [int(rng.integers(0, V // 2 - 9000)) * 64, int(rng.integers(3000, 9000)) * 16]
                    if i == 100:
                        args = [30000 * 64, 12000 * 16]
                g.ms.launch_enqueue(task, kg, args, 2, ids_ptr=dev[task, i].data_ptr(), n_ids=n_ids)
                o.launch_enqueue(task, ko, args, 2, ids=ids[task, i])
        for k, tl in enumerate(([(0, n_cmds), (1, n_cmds)], [(1, n_cmds), (0, n_cmds)], [(0, n_cmds), (1, n_cmds)])):
            po, pg = o.plan(tl), g.ms.plan(tl)
            if k == 0:
                assert pg.n_commands == 2 * n_cmds
            assert_same_plan(po, pg, tl)
            o.migrate()
            g.ms.migrate()
            pto, foo = o.state()
            ptg, fog = g.ms.state()
            assert np.array_equal(pto, ptg) and np.array_equal(foo, fog)
            n = min(po.covered_launches, 60)
            o.launch_retire(tl[0][0], n)
            g.ms.launch_retire(tl[0][0], n)
        bad = torch.tensor([3, V + 5, 9], dtype=torch.int32, device="cuda")
        g.ms.launch_enqueue(1, kg, [0, 16], 2, ids_ptr=bad.data_ptr(), n_ids=3)
        with pytest.raises(MSchedError) as e:
            g.ms.plan([(0, 2), (1, n_cmds + 5)])
        assert e.value.name == "E_RANGE"
    finally:
        g.close()
        o.close()


def test_a_prepared_list_with_a_bad_id_is_refused_by_every_plan(oracle_mod, monkeypatch):
    import torch
    from paper_2512_24637_amd import MSchedError
    monkeypatch.setenv("MSCHED_LIST_BINNED_MIN_IDS", "0")
    trace = explicit_trace([[[0]], [[1]]], 64, 16, timeslice=2, page_shift=6)
    g = GpuSide(trace)
    try:
        ms = g.ms
        kl = ms.kernel_register([Rule(RULE_LIST)])
        bad = torch.tensor([3, 400, 5], dtype=torch.int32, device="cuda")      # 400 >= V
        ms.launch_enqueue(1, kl, [], 0, ids_ptr=bad.data_ptr(), n_ids=3)
        for _ in range(3):                               # the list is prepared by the first plan, refused by all
            with pytest.raises(MSchedError) as e:
                ms.plan([(0, 1), (1, 2)])
            assert e.value.name == "E_RANGE"
        p = ms.plan([(0, 1)])                            # a timeline without that command is fine
        assert p.n_fetch == 1
    finally:
        g.close()


def test_a_refused_plan_leaves_nothing_behind_for_the_next_one(oracle_mod):
    """After E_WSET_TOO_LARGE the same queues planned with a timeline that fits give the oracle's plan (the
    repeat-region table of the refused attempt must not count as this plan's)."""
    from paper_2512_24637_amd import MSchedError
    trace = explicit_trace([[[0, 1, 2, 3], [4]], [[5, 6], [0, 1]]], 8, 3, timeslice=2, page_shift=6)
    g = GpuSide(trace)
    o = make_oracle(oracle_mod, trace, with_bytes=False)
    try:
        with pytest.raises(MSchedError) as e:
            g.ms.plan([(0, 2), (1, 2)])
        assert e.value.name == "E_WSET_TOO_LARGE"
        for tl in ([(1, 2), (0, 2)], [(1, 1)]):
            assert_same_plan(o.plan(tl), g.ms.plan(tl), tl)
    finally:
        g.close()
        o.close()


class _NoReadBack:
    """Drives the HIP path the way a scheduler would: counts from msched_plan, then msched_migrate at once - no list
    is read back and nothing waits for the stream in between."""

    def __init__(self, ms):
        self.ms = ms
        self.counts = []

    def plan(self, timeline):
        p = self.ms.plan(timeline)
        self.counts.append((p.n_fetch, p.n_evict, p.n_free_used, p.g_cut, p.covered_launches))
        return p

    def migrate(self):
        self.ms.migrate_only()

    def launch_retire(self, task, n):
        self.ms.launch_retire(task, n)


@pytest.mark.parametrize("cfg,kw", [(1, dict(seed=3)), (5, dict(scale=64, n_launches=100)),
                                    (4, dict(page_shift=12, layers=8, steps=16))])
def test_migrate_straight_after_plan_without_any_wait(oracle_mod, monkeypatch, cfg, kw):
    """msched_plan returns when the counts are known, while the kernels that fill the lists may still run; the
    migration queued behind them must find the lists complete.  Counts of every switch, and page table, frame
    owners, pool and host bytes at the end, against the oracle."""
    monkeypatch.setenv("MSCHED_LIST_BINNED_MIN_IDS", "0")
    trace = make_trace(cfg, **kw)
    g = GpuSide(trace)
    o = make_oracle(oracle_mod, trace, with_bytes=True)
    try:
        drv = _NoReadBack(g.ms)
        n = sum(1 for _ in run_schedule(trace, drv))
        expected = []
        for rec in run_schedule(trace, o):
            expected.append((rec.plan.n_fetch, rec.plan.n_evict, rec.plan.n_free_used, rec.plan.g_cut, rec.plan.covered_launches))
        assert n == len(expected) and drv.counts == expected
        pto, foo = o.state()
        ptg, fog = g.ms.state()
        assert np.array_equal(pto, ptg) and np.array_equal(foo, fog)
        assert np.array_equal(o.pool_words, g.pool_words()), "pool bytes"
        assert np.array_equal(o.host_words, g.host_words()), "host bytes"
    finally:
        g.close()
        o.close()
