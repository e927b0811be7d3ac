"""Pins for the oracle's early-execution functions (Sec. 6.3 of the paper: pages migrate in predicted access
order and a kernel starts as soon as the pages it depends on are resident).  Expected values are rebuilt here
from command page sets and residency, without the oracle's lists or next-use table."""
import numpy as np
import pytest

from workloads import make_trace, run_schedule
from workloads.harness import load_trace

NONE = 0xFFFFFFFF


def _schedule(oracle_mod, trace, with_bytes=False):
    o = oracle_mod.Oracle.for_trace(trace, with_bytes=with_bytes)
    load_trace(o, trace)
    return o


def _need_by_definition(o, rec, pt_before):
    """For each covered command g: the non-resident pages that commands 0..g of the incoming task use."""
    missing, need = set(), []
    for g in range(rec.n_launches):
        pages = o.command_pages(rec.task, rec.first_launch + g)
        missing |= {int(p) for p in pages if pt_before[p] == NONE}
        need.append(len(missing))
    return np.array(need, np.uint32), missing


@pytest.mark.parametrize("config,kw", [(1, {}), (3, dict(scale=32, n_launches=192)), (4, dict(page_shift=15, n_launches=256))])
def test_need_counts_the_missing_pages_of_the_commands_so_far(oracle_mod, config, kw):
    trace = make_trace(config, **kw)
    o = _schedule(oracle_mod, trace)
    pt_before, _ = o.state()
    seen = 0
    # the harness calls migrate() right after plan(); need[] belongs to the pending plan, so drive by hand
    cursor = [0] * trace.n_tasks
    for step in range(12):
        t = step % trace.n_tasks
        if cursor[t] >= len(trace.tasks[t]):
            continue
        tl = [((t + k) % trace.n_tasks, trace.timeslice) for k in range(trace.n_tasks)
              if cursor[(t + k) % trace.n_tasks] < len(trace.tasks[(t + k) % trace.n_tasks])]
        plan = o.plan(tl)
        need = o.ready_need(plan.g_cut)

        class Rec:
            task, first_launch, n_launches = t, cursor[t], plan.covered_launches
        want, missing = _need_by_definition(o, Rec, pt_before)
        assert np.array_equal(need, want), (config, step)
        assert need.size == 0 or need[-1] == plan.n_fetch
        assert set(plan.fetch_pages.tolist()) == missing
        # landing a prefix of need[g] entries makes commands 0..g runnable, one entry less does not
        landed = 0
        for g in sorted({0, plan.g_cut // 2, plan.g_cut - 1} & set(range(plan.g_cut))):
            if landed == plan.n_fetch:
                break                                          # an empty or finished plan: nothing left to land
            if need[g] > landed and (g == 0 or need[g] > need[g - 1]):
                o.migrate_prefix(need[g] - 1)
                pt, _ = o.state()
                assert any(pt[p] == NONE for gg in range(g + 1) for p in o.command_pages(t, cursor[t] + gg))
            o.migrate_prefix(need[g])
            landed = int(need[g])
            pt, _ = o.state()
            assert all(pt[p] != NONE for gg in range(g + 1) for p in o.command_pages(t, cursor[t] + gg))
            seen += 1
        if landed < plan.n_fetch or plan.n_fetch == 0:
            o.migrate_prefix(plan.n_fetch)
        pt_before, _ = o.state()
        o.launch_retire(t, plan.covered_launches)
        cursor[t] += plan.covered_launches
    assert seen >= 6
    o.close()


def test_prefix_by_prefix_equals_the_whole_migration(oracle_mod):
    trace = make_trace(1)
    a, b = _schedule(oracle_mod, trace, with_bytes=True), _schedule(oracle_mod, trace, with_bytes=True)
    for o in (a, b):
        o.host_words[:] = np.arange(o.host_words.size, dtype=np.uint64).reshape(o.host_words.shape) * np.uint64(2654435761)
        o.pool_words[:] = np.uint64(7)
    rng = np.random.default_rng(5)
    n = 0
    for ra, rb_plan in zip(run_schedule(trace, a, max_plans=30), _prefix_runner(trace, b, rng, max_plans=30)):
        assert np.array_equal(ra.plan.fetch_pages, rb_plan.fetch_pages)
        pa, fa = a.state()
        pb, fb = b.state()
        assert np.array_equal(pa, pb) and np.array_equal(fa, fb)
        assert np.array_equal(a.pool_words, b.pool_words) and np.array_equal(a.host_words, b.host_words)
        n += 1
    assert n >= 15                                           # the schedule has about 20 context switches
    a.close()
    b.close()


def _prefix_runner(trace, o, rng, max_plans):
    """run_schedule with migrate() replaced by random prefix steps."""
    class Stepwise:
        def __getattr__(self, name):
            return getattr(o, name)

        def migrate(self):
            done, total = 0, self.last.n_fetch
            while done < total:
                done = min(total, done + int(rng.integers(1, 6)))
                o.migrate_prefix(done)
            if total == 0:
                o.migrate_prefix(0)

        def plan(self, tl):
            self.last = o.plan(tl)
            return self.last
    for rec in run_schedule(trace, Stepwise(), max_plans=max_plans):
        yield rec.plan


def test_prefix_argument_errors(oracle_mod):
    trace = make_trace(1)
    o = _schedule(oracle_mod, trace)
    with pytest.raises(oracle_mod.OracleError):
        o.migrate_prefix(0)                                   # nothing planned
    plan = o.plan([(0, trace.timeslice)])
    assert plan.n_fetch > 2
    with pytest.raises(oracle_mod.OracleError):
        o.migrate_prefix(plan.n_fetch + 1)
    o.migrate_prefix(2)
    with pytest.raises(oracle_mod.OracleError):
        o.migrate_prefix(1)                                   # cannot go back
    with pytest.raises(oracle_mod.OracleError):
        o.migrate()                                           # a started prefix is finished the same way
    o.migrate_prefix(plan.n_fetch)
    with pytest.raises(oracle_mod.OracleError):
        o.migrate_prefix(plan.n_fetch)                        # done
    o.close()
