"""Early execution on the HIP path (msched_set_early_start / msched_plan_ready_need / msched_progress;
paper Sec. 6.3): need[] bit-exact against the oracle, the same final state as a plain migration, and, while a
migration is still in flight, every entry below the published `landed` mark already holds its bytes."""
import time

import numpy as np
import pytest

from workloads import make_trace, run_schedule
from gpu_common import GpuSide, make_oracle, assert_same_plan

pytestmark = pytest.mark.gpu
NONE = 0xFFFFFFFF


class _WithNeed:
    """Records need[] of every plan before the driver migrates it."""

    def __init__(self, impl, need_of):
        self.impl, self.need_of, self.need = impl, need_of, None

    def __getattr__(self, name):
        return getattr(self.impl, name)

    def plan(self, tl):
        p = self.impl.plan(tl)
        self.need = self.need_of(p)
        return p


@pytest.mark.parametrize("config,kw", [(1, {}), (3, dict(scale=16, n_launches=480)), (4, dict(page_shift=16, n_launches=512)),
                                       (5, dict(scale=64, n_launches=100))])
def test_need_and_final_state_match_the_oracle(oracle_mod, config, kw):
    trace = make_trace(config, **kw)
    g = GpuSide(trace)
    g.ms.set_early_start(True)
    o = make_oracle(oracle_mod, trace, with_bytes=True)
    wo = _WithNeed(o, lambda p: o.ready_need(p.g_cut))
    wg = _WithNeed(g.ms, lambda p: g.ms.ready_need(p))
    n = 0
    try:
        for ro, rg in zip(run_schedule(trace, wo, max_plans=40), run_schedule(trace, wg, max_plans=40)):
            where = (trace.name, "plan", ro.index)
            assert_same_plan(ro.plan, rg.plan, where)
            assert np.array_equal(wo.need, wg.need), (where, "need")
            g.torch.cuda.synchronize()
            assert g.ms.progress() == rg.plan.n_fetch or rg.plan.n_fetch == 0, where
            pto, foo = o.state()
            ptg, fog = g.ms.state()
            assert np.array_equal(pto, ptg) and np.array_equal(foo, fog), where
            if n % 4 == 0:
                assert np.array_equal(o.pool_words, g.pool_words()), (where, "pool bytes")
                assert np.array_equal(o.host_words, g.host_words()), (where, "host bytes")
            n += 1
        assert n >= 8
    finally:
        g.close()
        o.close()


def test_need_is_refused_without_early_start(oracle_mod):
    from paper_2512_24637_amd import MSchedError
    trace = make_trace(1)
    g = GpuSide(trace)
    try:
        p = g.ms.plan([(0, trace.timeslice)])
        with pytest.raises(MSchedError) as e:
            g.ms.ready_need(p)
        assert e.value.code == -5
        assert g.ms.progress() == 0
        g.ms.migrate()
        g.ms.set_early_start(True)
        g.ms.launch_retire(0, p.covered_launches)
        p = g.ms.plan([(1, trace.timeslice)])
        need = g.ms.ready_need(p)
        assert need.size == p.covered_launches and need[-1] == p.n_fetch
        assert g.ms.progress() == 0                      # planned, not migrated yet
        g.ms.migrate()
        g.torch.cuda.synchronize()
        assert g.ms.progress() == p.n_fetch
    finally:
        g.close()


def test_landed_entries_hold_their_bytes_while_the_migration_runs():
    """LLM-decode schedule with 512 KiB pages (several gigabytes per switch, every layer's weights needed by a
    later launch): poll the progress mark during the copy and read, on a second stream, the first and last
    word of every frame below it.  They must equal the page's words in the host store, which a fetch never
    changes.  The mark must also move while the copy runs, roughly in step with it."""
    import torch
    trace = make_trace(4, page_shift=19, steps=16)
    g = GpuSide(trace)
    g.ms.set_early_start(True)
    side = torch.cuda.Stream()
    main = torch.cuda.current_stream()
    try:
        impl = _SampledMigrate(g, side, main, g.host)
        with torch.cuda.stream(side):                          # torch loads its gather kernels on first use: not mid-copy
            idx = torch.zeros(4, dtype=torch.int64, device=g.device)
            torch.stack([g.pool[idx, 0], g.pool[idx, -1]], 1).cpu()
        torch.cuda.synchronize()
        switches = sum(1 for _ in run_schedule(trace, impl, max_plans=6))
        assert switches == 6
        assert _SampledMigrate.entries_checked > 10000
        assert _SampledMigrate.in_flight >= 20, "the progress mark was hardly ever read while a copy was running"
        # a launch a quarter of the way into the fetch list was ready well before the copy ended
        assert _SampledMigrate.early_fraction and max(_SampledMigrate.early_fraction) < 0.6, _SampledMigrate.early_fraction
    finally:
        g.close()


class _SampledMigrate:
    in_flight = 0
    entries_checked = 0
    early_fraction = []          # per switch: when the first quarter of the fetch list had landed / when all had

    def __init__(self, g, side, main, host):
        self.g, self.side, self.main, self.host = g, side, main, host
        _SampledMigrate.in_flight = 0
        _SampledMigrate.entries_checked = 0
        _SampledMigrate.early_fraction = []

    def __getattr__(self, name):
        return getattr(self.g.ms, name)

    def plan(self, tl):
        self.last = self.g.ms.plan(tl)
        return self.last

    def migrate(self):
        import torch
        g, p = self.g, self.last
        need = g.ms.ready_need(p)
        pages, frames = p.fetch_pages.astype(np.int64), p.fetch_frames.astype(np.int64)
        slots = np.asarray(g.ms.slot_of(pages), np.int64)
        frames_dev = torch.from_numpy(frames).to(g.device)
        g.torch.cuda.synchronize()
        g.ms.migrate()
        done, samples = 0, []
        marks = sorted(set(int(x) for x in need if x > 0))
        t0 = time.monotonic()
        deadline, t_quarter = t0 + 30.0, None
        while done < p.n_fetch:
            assert time.monotonic() < deadline, ("progress stuck at", done, "of", p.n_fetch)
            landed = g.ms.progress()
            if t_quarter is None and landed >= p.n_fetch // 4:
                t_quarter = time.monotonic() - t0
            busy = not self.main.query()
            ready = [m for m in marks if done < m <= landed]
            if not ready:
                if not busy:
                    assert g.ms.progress() == p.n_fetch       # the copy has ended: everything has landed
                continue
            upto = ready[-1]                                  # commands up to this mark may start now
            with torch.cuda.stream(self.side):
                idx = frames_dev[done:upto]
                first_last = torch.stack([g.pool[idx, 0], g.pool[idx, -1]], 1).cpu()
            samples.append((done, upto, first_last, busy))
            done = upto
        g.torch.cuda.synchronize()
        if p.n_fetch >= 1000:
            _SampledMigrate.early_fraction.append(t_quarter / (time.monotonic() - t0))
        for lo, hi, got, busy in samples:
            want = np.stack([self.host[torch.from_numpy(slots[lo:hi]), 0].numpy(),
                             self.host[torch.from_numpy(slots[lo:hi]), -1].numpy()], 1)
            assert np.array_equal(got.numpy(), want), ("entries", lo, hi, "read before they had landed")
            _SampledMigrate.entries_checked += hi - lo
            _SampledMigrate.in_flight += int(busy)


def test_device_side_gates_release_consumers_when_their_pages_are_in():
    """msched_gate_enqueue: gates for the first, a middle and the last covered command on a second stream, each
    followed by a kernel that reads the frames of the fetch entries the command needs while the migration is still
    running on the context's stream; every gate reports "resident", later gates report later times, the reads
    find the pages' words, and the first command's gate opens while the migration is still in flight.  A gate with
    a microsecond to live, queued behind the start of a migration of hundreds of megabytes, gives up (status 2)
    and its stream moves on."""
    import torch
    from workloads import page_words
    from paper_2512_24637_amd import MSchedError
    trace = make_trace(4, page_shift=16, n_launches=512)     # decode: every launch of a step needs one more layer
    g = GpuSide(trace)
    try:
        g.ms.set_early_start(True)
        side = torch.cuda.Stream()
        wpp = trace.page_bytes // 8
        seen_in_flight = gave_up = 0
        for sw in range(4):
            t = sw % trace.n_tasks
            p = g.ms.plan([((t + k) % trace.n_tasks, trace.timeslice) for k in range(trace.n_tasks)])
            need = g.ms.ready_need(p)
            with pytest.raises(MSchedError):                  # not before its migration
                g.ms.gate_enqueue(p, 0, side.cuda_stream)
            fetch_pages, fetch_frames = p.fetch_pages.copy(), p.fetch_frames.copy()
            frames_dev = torch.from_numpy(fetch_frames.astype(np.int64)).cuda()
            last = p.covered_launches - 1
            torch.cuda.synchronize()
            g.ms.migrate_only(p)
            if sw == 1:
                g.ms.gate_enqueue(p, last, side.cuda_stream, timeout_us=1)
                side.synchronize()
                st, ms = g.ms.gate_result(last)
                assert st in (1, 2) and (st == 1 or ms == 0.0)
                gave_up += st == 2
            picks = sorted({0, p.covered_launches // 3, last})
            got = []
            with torch.cuda.stream(side):
                for j, gi in enumerate(picks):
                    g.ms.gate_enqueue(p, gi, side.cuda_stream)
                    lo = max(0, int(need[gi]) - 64)
                    got.append((gi, lo, g.pool[frames_dev[lo:int(need[gi])]].clone()))   # runs behind the gate
                    if j == 0:
                        side.synchronize()
                        seen_in_flight += not g.stream.query()
            side.synchronize()
            results = [g.ms.gate_result(gi) for gi in picks]
            assert all(st == 1 for st, _ in results), results
            times = [ms for _, ms in results]
            assert times == sorted(times), times
            for gi, lo, words in got:
                want = page_words(fetch_pages[lo:int(need[gi])], wpp)
                assert np.array_equal(words.cpu().numpy().view(np.uint64), want), (sw, gi)
            torch.cuda.synchronize()
            assert g.ms.progress() == p.n_fetch
            g.ms.launch_retire(t, p.covered_launches)
        assert seen_in_flight >= 2, "the first command's gate should open while the migration is still running"
        assert gave_up == 1
    finally:
        g.close()
