"""Seeded generators for the synthetic schedules.

Each stands in for one of the paper's workload classes (Sec. 7: micro-benchmark,
scientific computing, DNN training, LLM decoding; the fifth stresses planning
with sparse gathers, which the paper leaves to demand paging).  Shapes follow
the benchmark configuration; `page_shift`, `scale` and the per-config count
overrides shrink a schedule for CPU-sized tests without changing its page
structure.

Only launch arguments and templates are produced.  Page sets are never
computed here.
"""
from typing import Optional

import numpy as np

from .trace import (RULE_FIXED, RULE_LINEAR, RULE_STRIDED, RULE_LIST, Rule,
                    Trace, CommandBuilder)

CONFIG_NAMES = {
    1: "c1-tiny-round-robin",
    2: "c2-stencil-sweep",
    3: "c3-dl-training",
    4: "c4-llm-decode",
    5: "c5-planning-stress",
    6: "c6-priority-colocation",
}

KiB = 1 << 10
MiB = 1 << 20


def _ragged_extent(rng, first_page, n_pages, page_bytes, elem):
    """Pick a byte range whose outward page alignment is exactly
    [first_page, first_page + n_pages): a ragged start inside the first page and
    a ragged end inside the last one, both multiples of `elem`."""
    lead = int(rng.integers(0, page_bytes // elem)) * elem
    if n_pages == 1:
        room = page_bytes - lead
        size = int(rng.integers(1, room // elem + 1)) * elem
    else:
        tail_room = page_bytes // elem
        tail = int(rng.integers(1, tail_room + 1)) * elem        # bytes used in the last page
        size = (page_bytes - lead) + (n_pages - 2) * page_bytes + tail
    base = first_page * page_bytes + lead
    return base, size


def _c1(seed, page_shift, scale, n_launches):
    page_shift = 16 if page_shift is None else page_shift
    P = 1 << page_shift
    n_tasks, pages_per_task, slice_len = 3, 128, 10
    n_launches = 200 if n_launches is None else n_launches
    rng = np.random.default_rng([seed, 1])
    # k0: scale(A, N); k1: axpy(A, B, NA, NB); k2: gemm-like(A, B, C, NA, NB, MC, KC)
    kernels = [
        [Rule(RULE_LINEAR, 0, (1,), 4)],
        [Rule(RULE_LINEAR, 0, (2,), 4), Rule(RULE_LINEAR, 1, (3,), 8)],
        [Rule(RULE_LINEAR, 0, (3,), 4), Rule(RULE_LINEAR, 1, (4,), 4),
         Rule(RULE_LINEAR, 2, (5, 6), 2)],
    ]
    builders = [CommandBuilder() for _ in range(n_tasks)]
    for j in range(n_launches):
        task = (j // slice_len) % n_tasks
        n_rules = int(rng.integers(1, 4))
        bases, counts = [], []
        for r in range(n_rules):
            length = int(rng.integers(4, 65))
            start = int(rng.integers(0, pages_per_task - length + 1)) + task * pages_per_task
            if n_rules == 3 and r == 2:
                k_dim = int(rng.choice([64, 128, 256]))
                elem = 2 * k_dim
                base, size = _ragged_extent(rng, start, length, P, elem)
                bases.append(base)
                counts.extend([size // elem, k_dim])
            else:
                elem = 8 if (n_rules == 2 and r == 1) else 4
                base, size = _ragged_extent(rng, start, length, P, elem)
                bases.append(base)
                counts.append(size // elem)
        builders[task].add(n_rules - 1, bases + counts, latency=1)
    return Trace(
        name=CONFIG_NAMES[1], page_shift=page_shift,
        n_virtual_pages=n_tasks * pages_per_task, n_frames=256, timeslice=slice_len,
        kernels=kernels, tasks=[b.build() for b in builders],
        n_slots=n_tasks * pages_per_task,
        notes="3 equal tasks, 1-3 linear-size ranges of 4-64 pages per launch")


def _c2(seed, page_shift, scale, n_launches):
    page_shift = 21 if page_shift is None else page_shift
    P = 1 << page_shift
    n_tasks, arrays, pages_per_array, slice_len = 4, 3, 128, 25
    per_task = 500 if n_launches is None else n_launches
    array_bytes = pages_per_array * P               # 256 MiB at 2 MiB pages
    kernels = [[Rule(RULE_FIXED, 0, (), array_bytes), Rule(RULE_FIXED, 1, (), array_bytes),
                Rule(RULE_FIXED, 2, (), array_bytes)]]
    tasks = []
    for t in range(n_tasks):
        b = CommandBuilder()
        base = [(t * arrays + a) * array_bytes for a in range(arrays)]
        for it in range(per_task):
            # read two arrays, write the third, rotating (ping-pong sweep)
            r = it % 3
            b.add(0, [base[r], base[(r + 1) % 3], base[(r + 2) % 3]], latency=1)
        tasks.append(b.build())
    V = n_tasks * arrays * pages_per_array
    return Trace(name=CONFIG_NAMES[2], page_shift=page_shift, n_virtual_pages=V,
                 n_frames=1024, timeslice=slice_len, kernels=kernels, tasks=tasks, n_slots=V,
                 notes="4 tasks x 3 arrays of 128 pages, every launch touches all three")


def _c3(seed, page_shift, scale, n_launches, layers=48, iterations=20):
    page_shift = 16 if page_shift is None else page_shift
    P = 1 << page_shift
    rng = np.random.default_rng([seed, 3])
    s = max(1, int(scale))
    cols = 4096
    batch, feat = 4096 // s, 4096                    # activation = 2*batch*feat bytes (32 MiB / s)
    act_bytes = 2 * batch * feat
    fwd = [Rule(RULE_LINEAR, 0, (3, 4), 2), Rule(RULE_LINEAR, 1, (5, 6), 2),
           Rule(RULE_LINEAR, 2, (5, 6), 2)]
    bwd = [Rule(RULE_LINEAR, 0, (6, 7), 2), Rule(RULE_LINEAR, 1, (6, 7), 2),
           Rule(RULE_LINEAR, 2, (8, 9), 2), Rule(RULE_LINEAR, 3, (8, 9), 2),
           Rule(RULE_FIXED, 4, (), act_bytes), Rule(RULE_FIXED, 5, (), act_bytes)]
    kernels = [fwd, bwd]
    tasks, cursor = [], 0                            # cursor: next free byte (page aligned)

    allocations = []

    def alloc(nbytes):
        nonlocal cursor
        addr = cursor
        cursor += -(-nbytes // P) * P
        allocations.append((addr, nbytes))
        return addr

    for t in range(2):
        rows = rng.integers(8192 // s, 24576 // s + 1, size=layers)   # 64..192 MiB of bf16 / s
        W = [alloc(int(r) * cols * 2) for r in rows]
        dW = [alloc(int(r) * cols * 2) for r in rows]
        A = [alloc(act_bytes) for _ in range(layers + 1)]             # A[0] is the input batch
        G = [alloc(act_bytes), alloc(act_bytes)]
        b = CommandBuilder()
        for it in range(iterations):
            for l in range(layers):
                b.add(0, [W[l], A[l], A[l + 1], int(rows[l]), cols, batch, feat], latency=1)
            for l in reversed(range(layers)):
                b.add(1, [W[l], dW[l], A[l + 1], A[l], G[l % 2], G[(l + 1) % 2],
                          int(rows[l]), cols, batch, feat], latency=1)
        tasks.append(b.build())
    V = cursor // P
    return Trace(name=CONFIG_NAMES[3], page_shift=page_shift, n_virtual_pages=V,
                 n_frames=V // 2, timeslice=2 * layers, kernels=kernels, tasks=tasks, n_slots=V,
                 notes=f"2 tasks, {layers} layers, fwd+bwd per iteration, pool = half the footprint",
                 allocations=np.asarray(allocations, np.uint64))


def _c4(seed, page_shift, scale, n_launches, layers=32, steps=256, full_backing=False):
    page_shift = 21 if page_shift is None else page_shift
    P = 1 << page_shift
    unit = P / (2 * MiB)                             # byte sizes scale with the page size
    attn_bytes = int(64 * MiB * unit)
    ffn_bytes = int(336 * MiB * unit)
    token_bytes = int(8 * KiB * unit)                # one token of K (or V): 32 heads x 128 x bf16
    max_tokens, batch, start_ctx, steps_per_slice = 4096, 8, 384, 4
    final_ctx = start_ctx + 256                      # the layout is sized for the full 256-step run
    stride = token_bytes * max_tokens                # one sequence's slab: 32 MiB
    attn = [Rule(RULE_FIXED, 0, (), attn_bytes),
            Rule(RULE_STRIDED, 1, (3,), token_bytes, (4,), token_bytes, (5,), 1),
            Rule(RULE_STRIDED, 2, (3,), token_bytes, (4,), token_bytes, (5,), 1)]
    ffn = [Rule(RULE_FIXED, 0, (), ffn_bytes)]
    kernels = [attn, ffn]
    tasks, cursor = [], 0
    slot_pages = []                                   # page ids that own a backing slot

    allocations = []

    def alloc(nbytes):
        nonlocal cursor
        addr = cursor
        cursor += -(-nbytes // P) * P
        allocations.append((addr, nbytes))
        return addr

    for t in range(2):
        Wa, Wf, Kc, Vc = [], [], [], []
        for l in range(layers):
            Wa.append(alloc(attn_bytes))
            Wf.append(alloc(ffn_bytes))
            slot_pages.append(np.arange(Wa[-1] // P, (Wf[-1] + ffn_bytes + P - 1) // P))
        for l in range(layers):
            for cache in (Kc, Vc):
                base = alloc(stride * batch)
                cache.append(base)
                used = -(-(final_ctx * token_bytes) // P)       # pages a sequence can ever touch
                for bi in range(batch):
                    first = (base + bi * stride) // P
                    slot_pages.append(np.arange(first, first + used))
        b = CommandBuilder()
        for s_ in range(steps):
            L = start_ctx + 1 + s_
            for l in range(layers):
                b.add(0, [Wa[l], Kc[l], Vc[l], L, max_tokens, batch], latency=1)
                b.add(1, [Wf[l]], latency=1)
        tasks.append(b.build())
    V = cursor // P
    pages = np.unique(np.concatenate(slot_pages))
    host_slot = np.full(V, 0xFFFFFFFF, np.uint32)
    host_slot[pages] = np.arange(pages.size, dtype=np.uint32)
    if full_backing:                                 # every page of every buffer can be paged (allocation-granularity ablation)
        host_slot, pages = None, np.arange(V)
    n_frames = int(8192 * layers / 32)
    return Trace(name=CONFIG_NAMES[4], page_shift=page_shift, n_virtual_pages=V,
                 n_frames=n_frames, timeslice=steps_per_slice * 2 * layers, kernels=kernels,
                 tasks=tasks, host_slot=host_slot, n_slots=int(pages.size),
                 notes=f"2 decoders, {layers} layers, KV grows one token per step",
                 allocations=np.asarray(allocations, np.uint64))


def _zipf_cdf(n_items, alpha):
    w = np.arange(1, n_items + 1, dtype=np.float64) ** (-alpha)
    cdf = np.cumsum(w)
    return cdf / cdf[-1]


def _zipf_ranks(rng, cdf, size):
    return np.minimum(np.searchsorted(cdf, rng.random(size)), cdf.size - 1)


def _c5(seed, page_shift, scale, n_launches):
    page_shift = 12 if page_shift is None else page_shift
    P = 1 << page_shift
    s = max(1, int(scale))
    n_tasks, slice_len = 8, 50
    private = (1 << 20) // s
    table = (2 << 20) // s
    n_ids = 20000 // s
    lo, hi = max(1, 1024 // s), max(2, 16384 // s)
    per_task = (625 if n_launches is None else n_launches)
    rng = np.random.default_rng([seed, 5])
    perm = rng.permutation(table).astype(np.uint32)
    cdf = _zipf_cdf(table, 1.1)
    table_base = n_tasks * private
    kernels = [[Rule(RULE_LINEAR, 0, (2,), 4), Rule(RULE_LINEAR, 1, (3,), 4),
                Rule(RULE_LIST)]]
    builders = [CommandBuilder() for _ in range(n_tasks)]
    pools, off = [], 0
    for t in range(n_tasks):
        for j in range(per_task):
            args = []
            counts = []
            for r in range(2):
                length = int(rng.integers(lo, hi + 1))
                start = int(rng.integers(0, private - length + 1)) + t * private
                base, size = _ragged_extent(rng, start, length, P, 4)
                args.append(base)
                counts.append(size // 4)
            ranks = _zipf_ranks(rng, cdf, n_ids)
            pools.append(perm[ranks] + np.uint32(table_base))
            builders[t].add(0, args + counts, latency=1, ids_off=off, n_ids=n_ids)
            off += n_ids
    V = table_base + table
    return Trace(name=CONFIG_NAMES[5], page_shift=page_shift, n_virtual_pages=V,
                 n_frames=(4 << 20) // s, timeslice=slice_len, kernels=kernels,
                 tasks=[b.build() for b in builders],
                 ids_pool=(np.concatenate(pools).astype(np.uint32) if pools else np.zeros(0, np.uint32)),
                 n_slots=V,
                 notes="8 tasks, 2 dense ranges + Zipf(1.1) page-id gather over a shared table")


def _c6(seed, page_shift, scale, n_launches, rt_layers=50, be_layers=40, requests=12, be_iterations=6):
    """Real-time inference beside best-effort training under a priority policy (the paper's colocation
    test T): task 0 serves requests of `rt_layers` launches, one layer each, and preempts task 1, which
    trains (forward + backward over `be_layers` layers).  The real-time model takes a third of the footprint
    and the pool holds 8/9 of it, the paper's 6 GB + 12 GB on a 16 GB card.  Launch latencies (ticks of a
    microsecond) follow the bytes a launch touches, with seeded jitter, as profiled latencies would."""
    page_shift = 16 if page_shift is None else page_shift
    P = 1 << page_shift
    rng = np.random.default_rng([seed, 6])
    s = max(1, int(scale))
    cols = 4096
    batch, feat = 2048 // s, 4096
    act_bytes = 2 * batch * feat                     # 16 MiB / s
    infer = [Rule(RULE_LINEAR, 0, (3, 4), 2), Rule(RULE_LINEAR, 1, (5, 6), 2), Rule(RULE_LINEAR, 2, (5, 6), 2)]
    fwd = infer
    bwd = [Rule(RULE_LINEAR, 0, (6, 7), 2), Rule(RULE_LINEAR, 1, (6, 7), 2),
           Rule(RULE_LINEAR, 2, (8, 9), 2), Rule(RULE_LINEAR, 3, (8, 9), 2),
           Rule(RULE_FIXED, 4, (), act_bytes), Rule(RULE_FIXED, 5, (), act_bytes)]
    kernels = [infer, fwd, bwd]
    cursor = 0

    allocations = []

    def alloc(nbytes):
        nonlocal cursor
        addr = cursor
        cursor += -(-nbytes // P) * P
        allocations.append((addr, nbytes))
        return addr

    def ticks(nbytes):                               # about 1 us per 2 MiB touched at full size, +-25 %
        return max(1, int(nbytes * s / (2 * MiB) * rng.uniform(0.75, 1.25)))

    # real-time task: weights 32..160 MiB / s per layer, two activation buffers reused by every layer
    rows = rng.integers(4096 // s, 20480 // s + 1, size=rt_layers)
    W = [alloc(int(r) * cols * 2) for r in rows]
    A = [alloc(act_bytes), alloc(act_bytes)]
    rt = CommandBuilder()
    for _ in range(requests):
        for l in range(rt_layers):
            rt.add(0, [W[l], A[l % 2], A[(l + 1) % 2], int(rows[l]), cols, batch, feat],
                   latency=ticks(int(rows[l]) * cols * 2 + 2 * act_bytes))
    rt_pages = cursor // P
    # best-effort task: training, twice the real-time footprint
    rows = rng.integers(8192 // s, 24576 // s + 1, size=be_layers)
    W = [alloc(int(r) * cols * 2) for r in rows]
    dW = [alloc(int(r) * cols * 2) for r in rows]
    A = [alloc(act_bytes) for _ in range(be_layers + 1)]
    G = [alloc(act_bytes), alloc(act_bytes)]
    be = CommandBuilder()
    for _ in range(be_iterations):
        for l in range(be_layers):
            be.add(1, [W[l], A[l], A[l + 1], int(rows[l]), cols, batch, feat],
                   latency=ticks(int(rows[l]) * cols * 2 + 2 * act_bytes))
        for l in reversed(range(be_layers)):
            be.add(2, [W[l], dW[l], A[l + 1], A[l], G[l % 2], G[(l + 1) % 2], int(rows[l]), cols, batch, feat],
                   latency=ticks(2 * int(rows[l]) * cols * 2 + 4 * act_bytes))
    V = cursor // P
    tasks = [rt.build(), be.build()]
    request_ticks = int(tasks[0].latency[:rt_layers].sum())
    return Trace(name=CONFIG_NAMES[6], page_shift=page_shift, n_virtual_pages=V, n_frames=V * 8 // 9,
                 timeslice=request_ticks, kernels=kernels, tasks=tasks, n_slots=V,
                 notes=f"real-time inference ({rt_pages} pages) preempting best-effort training ({V - rt_pages} pages)",
                 policy={"kind": "priority", "rt_task": 0, "be_task": 1, "request_launches": rt_layers,
                         "period": 4 * request_ticks, "be_quantum": 4 * request_ticks},
                 allocations=np.asarray(allocations, np.uint64))


def make_trace(config: int, seed: int = 0, page_shift: Optional[int] = None, scale: int = 1,
               n_launches: Optional[int] = None, **kw) -> Trace:
    """Build schedule `config` (1..6).

    page_shift  override the page size (byte sizes of c2/c4 scale with it, so
                the page structure is unchanged)
    scale       integer divisor for the size-like parameters of c3/c5
    n_launches  launches per task (total for c1) instead of the full count
    """
    gen = {1: _c1, 2: _c2, 3: _c3, 4: _c4, 5: _c5, 6: _c6}[config]
    return gen(seed, page_shift, scale, n_launches, **kw)
