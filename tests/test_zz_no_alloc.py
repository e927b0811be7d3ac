"""msched_pagetable_query_static (the entry point for callers that cannot allocate) against
msched_pagetable_query, through the C ABI, on a context with a part-resident page table
(needs an MI355X)."""
import numpy as np
import pytest

from workloads import make_trace, run_schedule
from gpu_common import GpuSide

pytestmark = pytest.mark.gpu


def test_static_query_equals_the_allocating_query_on_two_calls_in_a_row():
    from paper_2512_24637_amd import MSchedError
    from paper_2512_24637_amd.binding import QUERY_STATIC_MAX
    trace = make_trace(5, scale=64, n_launches=100)          # 160 Ki pages, a quarter of them resident after a few switches
    g = GpuSide(trace)
    try:
        for _ in run_schedule(trace, g.ms, max_plans=5):
            pass
        V = trace.n_virtual_pages
        rng = np.random.default_rng(7)
        first = rng.integers(0, V, size=QUERY_STATIC_MAX, dtype=np.uint64)      # the maximum size
        second = rng.integers(0, V, size=777, dtype=np.uint64)                  # then a smaller, ragged one
        for ids in (first, second, first[:1], np.zeros(0, np.uint64)):
            want = g.ms.pagetable_query(ids)
            got = g.ms.pagetable_query_static(ids)
            assert np.array_equal(want, got)
        pt, _ = g.ms.state()
        assert np.array_equal(g.ms.pagetable_query_static(second), pt[second.astype(np.int64)])
        assert (pt[first.astype(np.int64)] != 0xFFFFFFFF).any() and (pt[first.astype(np.int64)] == 0xFFFFFFFF).any()
        # beyond the array: refused, nothing done
        with pytest.raises(MSchedError) as err:
            g.ms.pagetable_query_static(np.zeros(QUERY_STATIC_MAX + 1, np.uint64))
        assert err.value.name == "E_TOO_LARGE"
        with pytest.raises(MSchedError) as err:
            g.ms.pagetable_query_static(np.array([V], np.uint64))
        assert err.value.name == "E_RANGE"
        # and the array is shared by every context on the GPU: a second context right after the first
        g2 = GpuSide(make_trace(1, seed=0, n_launches=60))
        try:
            for _ in run_schedule(g2.trace, g2.ms, max_plans=3):
                pass
            ids2 = np.arange(g2.trace.n_virtual_pages, dtype=np.uint64)
            assert np.array_equal(g2.ms.pagetable_query_static(ids2), g2.ms.pagetable_query(ids2))
            assert np.array_equal(g.ms.pagetable_query_static(second), g.ms.pagetable_query(second))
        finally:
            g2.close()
    finally:
        g.close()
