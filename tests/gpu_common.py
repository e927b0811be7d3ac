"""Shared plumbing of the GPU parity tests: device/pinned buffers for a trace, and the
lock-step comparison of the HIP path against the CPU oracle."""
import numpy as np

from workloads import run_schedule, page_words, stamp_of
from workloads.device import DeviceBuffers, POISON
from workloads.harness import load_trace

NONE = 0xFFFFFFFF


class GpuSide(DeviceBuffers):
    """Device buffers of a trace plus the MSched context that manages them."""

    def __init__(self, trace, preload=True):
        import torch
        from paper_2512_24637_amd import MSched
        super().__init__(trace)
        self.stream = torch.cuda.current_stream()
        self.ms = MSched(trace.page_shift, trace.n_virtual_pages, trace.n_frames, self.pool.data_ptr(),
                         self.host.data_ptr(), trace.n_slots, trace.host_slot,
                         stream=self.stream.cuda_stream, ids_pool_ptr=self.ids_ptr)
        if preload:
            load_trace(self.ms, trace)

    def close(self):
        self.torch.cuda.synchronize()
        self.ms.close()
        self.release()


def make_oracle(oracle_mod, trace, with_bytes, preload=True):
    o = oracle_mod.Oracle.for_trace(trace, with_bytes=with_bytes)
    if preload:
        load_trace(o, trace)
    if with_bytes:
        wpp = trace.page_bytes // 8
        pages = (np.arange(trace.n_virtual_pages) if trace.host_slot is None
                 else np.nonzero(trace.host_slot != NONE)[0])
        o.host_words[o.slot_of(pages)] = page_words(pages, wpp)
        o.pool_words[:] = np.uint64(POISON)
    return o


def assert_same_plan(po, pg, where):
    for f in ("n_fetch", "n_evict", "n_free_used", "g_cut", "g_end0", "n_commands", "covered_launches"):
        assert getattr(po, f) == getattr(pg, f), (where, f, getattr(po, f), getattr(pg, f))
    for f in ("fetch_pages", "fetch_frames", "evict_pages", "evict_frames"):
        a, b = getattr(po, f), getattr(pg, f)
        if not np.array_equal(a, b):
            bad = np.nonzero(a != b)[0]
            raise AssertionError((where, f, "first mismatch at", int(bad[0]), a[bad[:5]], b[bad[:5]]))


def lockstep(oracle_mod, trace, with_bytes=True, horizon="round", max_plans=None, bytes_every=1, log=None,
             lazy_slices=None, driver=None):
    """Run the oracle and the HIP path side by side and require identical plans, page
    tables, frame owners and (with_bytes) pool and host-store bytes after every switch.
    lazy_slices: enqueue launches only that many timeslices ahead of execution.
    driver: a scheduling policy other than round-robin, called as driver(trace, impl, max_plans) on an empty
    implementation (it registers kernels, tasks and launches itself)."""
    from workloads.harness import LazyLoader
    preload = lazy_slices is None and driver is None
    g = GpuSide(trace, preload=preload)
    o = make_oracle(oracle_mod, trace, with_bytes, preload=preload)
    lo = lg = None
    if lazy_slices is not None:
        lo, lg = LazyLoader(o, trace, lazy_slices), LazyLoader(g.ms, trace, lazy_slices)
    wpp = trace.page_bytes // 8
    n = 0
    try:
        if driver is not None:
            runs = zip(driver(trace, o, max_plans), driver(trace, g.ms, max_plans))
        else:
            runs = zip(run_schedule(trace, o, horizon=horizon, max_plans=max_plans, loader=lo),
                       run_schedule(trace, g.ms, horizon=horizon, max_plans=max_plans, loader=lg))
        for ro, rg in runs:
            where = (trace.name, "plan", ro.index, "task", ro.task)
            assert (ro.task, ro.first_launch, ro.timeline) == (rg.task, rg.first_launch, rg.timeline)
            assert_same_plan(ro.plan, rg.plan, where)
            idx, val = stamp_of(ro.plan.fetch_pages, ro.index, wpp)
            if with_bytes:
                o.pool_words[ro.plan.fetch_frames, idx] = val
            g.stamp(rg.plan.fetch_frames, idx, val)
            pto, foo = o.state()
            ptg, fog = g.ms.state()
            assert np.array_equal(pto, ptg), (where, "page table")
            assert np.array_equal(foo, fog), (where, "frame owner")
            if with_bytes and (n % bytes_every == 0):
                assert np.array_equal(o.pool_words, g.pool_words()), (where, "pool bytes")
                assert np.array_equal(o.host_words, g.host_words()), (where, "host bytes")
            n += 1
            if log:
                log(f"{trace.name} plan {ro.index}: fetch {ro.plan.n_fetch} evict {ro.plan.n_evict} ok")
        if with_bytes:
            assert np.array_equal(o.pool_words, g.pool_words())
            assert np.array_equal(o.host_words, g.host_words())
    finally:
        g.close()
        o.close()
    return n


def lockstep_sampled(oracle_mod, trace, n_sample=4096, max_plans=None, check_every=4, seed=1, log=None):
    """Full-size variant: plans, page table and frame owners are compared in full after every
    switch against the metadata-only oracle; bytes are compared on a seeded sample of pages whose
    expected contents (initial function of (page, word) plus every word the running task wrote)
    are tracked one by one on the CPU."""
    import torch
    g = GpuSide(trace)
    o = make_oracle(oracle_mod, trace, with_bytes=False)
    wpp = trace.page_bytes // 8
    rng = np.random.default_rng(seed)
    cand = g.pages_with_slot
    sample = np.sort(rng.choice(cand, size=min(n_sample, cand.size), replace=False))
    truth = page_words(sample, wpp)                       # [n_sample, wpp]
    slot_s = torch.from_numpy(np.asarray(o.slot_of(sample), np.int64))
    n = 0

    def check_bytes(where):
        pt = o.pagetable_query(sample)
        res = pt != NONE
        if res.any():
            rows = g.pool[torch.from_numpy(pt[res].astype(np.int64)).cuda()].cpu().numpy().view(np.uint64)
            assert np.array_equal(rows, truth[res]), (where, "sampled frames")
        if (~res).any():
            torch.cuda.synchronize()
            rows = g.host[slot_s[torch.from_numpy(~res)]].numpy().view(np.uint64)
            assert np.array_equal(rows, truth[~res]), (where, "sampled host slots")

    try:
        for ro, rg in zip(run_schedule(trace, o, max_plans=max_plans),
                          run_schedule(trace, g.ms, max_plans=max_plans)):
            where = (trace.name, "plan", ro.index, "task", ro.task)
            assert_same_plan(ro.plan, rg.plan, where)
            idx, val = stamp_of(rg.plan.fetch_pages, ro.index, wpp)
            g.stamp(rg.plan.fetch_frames, idx, val)
            pos = np.searchsorted(sample, ro.plan.fetch_pages)
            pos[pos == sample.size] = 0
            hit = sample[pos] == ro.plan.fetch_pages
            truth[pos[hit], idx[hit]] = val[hit]
            pto, foo = o.state()
            ptg, fog = g.ms.state()
            assert np.array_equal(pto, ptg), (where, "page table")
            assert np.array_equal(foo, fog), (where, "frame owner")
            if n % check_every == 0:
                check_bytes(where)
            n += 1
            if log:
                log(f"{trace.name} plan {ro.index}: fetch {ro.plan.n_fetch} evict {ro.plan.n_evict} "
                    f"covered {ro.plan.covered_launches}/{ro.plan.g_end0} ok")
        check_bytes((trace.name, "end"))
    finally:
        g.close()
        o.close()
    return n
