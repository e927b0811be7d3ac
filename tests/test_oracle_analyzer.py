"""Pins for the analyzer oracle (Sec. 5.2 "Memory analyzer" of the paper).  Expected values come from
the paper's two worked kernels, from an independent forward evaluation of the derived rules, and from
an exhaustive search over all (argument subset, coefficient) candidates written here."""
import itertools

import numpy as np
import pytest

from workloads.analyzer_inputs import make_batch, AnalyzerBatch, MAX_ARGS, FIXED, LINEAR, STRIDED


@pytest.fixture(scope="module")
def ana():
    from oracle import analyzer
    analyzer.build()
    return analyzer


def _single_kernel(n_args, ptr_mask, invocations):
    """invocations: list of (args list, [(start, len), ...])"""
    n_inv = len(invocations)
    max_iv = max(1, max(len(iv) for _, iv in invocations))
    args = np.zeros((1, n_inv, MAX_ARGS), np.uint64)
    iv = np.zeros((1, n_inv, max_iv, 2), np.uint64)
    n_iv = np.zeros((1, n_inv), np.uint32)
    for i, (a, rows) in enumerate(invocations):
        args[0, i, :len(a)] = a
        rows = sorted(rows)
        n_iv[0, i] = len(rows)
        for m, r in enumerate(rows):
            iv[0, i, m] = r
    return AnalyzerBatch(1, n_inv, max_iv, np.array([n_args], np.int32), np.array([ptr_mask], np.uint32), args, iv, n_iv,
                         [[]], np.zeros(1, np.uint32))


def _predict(rule, args):
    """Forward evaluation of a derived rule: the byte intervals it describes (independent of the oracle)."""
    kind, base_arg, s_idx, s_c, t_idx, t_c, c_idx, c_c = rule
    prod = lambda idx: int(np.prod([int(args[j]) for j in idx], dtype=object)) if idx else 1
    base = int(args[base_arg])
    size = s_c * prod(s_idx)
    if kind in (FIXED, LINEAR):
        return [(base, size)]
    return [(base + j * t_c * prod(t_idx), size) for j in range(c_c * prod(c_idx))]


def test_paper_vector_add_and_matrix_mul(ana):
    """vector_add(A,B,C,N): the three extents scale with N; matrix_mul(A,B,C,M,N,K): with M*K, K*N and
    M*N (Sec. 5.2, T2 example).  float32 elements."""
    A, B, Cc = 1 << 40, 2 << 40, 3 << 40
    inv = [([A + 64 * i, B + 128 * i, Cc + 256 * i, n], [(A + 64 * i, 4 * n), (B + 128 * i, 4 * n), (Cc + 256 * i, 4 * n)])
           for i, n in enumerate([1000, 4096, 77, 123456])]
    rules, un = ana.analyze(_single_kernel(4, 0b0111, inv))
    assert un[0] == 0
    assert rules[0] == [(LINEAR, 0, (3,), 4, (), 0, (), 0), (LINEAR, 1, (3,), 4, (), 0, (), 0), (LINEAR, 2, (3,), 4, (), 0, (), 0)]
    inv = []
    for i, (M, N, K) in enumerate([(64, 48, 80), (128, 128, 128), (7, 9, 11), (1000, 3, 17), (5, 600, 2)]):
        a = [A + 4 * i, B + 8 * i, Cc + 12 * i, M, N, K]
        inv.append((a, [(a[0], 4 * M * K), (a[1], 4 * K * N), (a[2], 4 * M * N)]))
    rules, un = ana.analyze(_single_kernel(6, 0b000111, inv))
    assert un[0] == 0
    assert rules[0] == [(LINEAR, 0, (3, 5), 4, (), 0, (), 0), (LINEAR, 1, (4, 5), 4, (), 0, (), 0),
                        (LINEAR, 2, (3, 4), 4, (), 0, (), 0)]


def test_invariant_size_is_fixed_whatever_the_arguments_do(ana):
    A = 5 << 40
    inv = [([A + 16 * i, n, m], [(A + 16 * i, 12345)]) for i, (n, m) in enumerate([(1, 2), (50, 7), (9, 9), (3, 1000)])]
    rules, un = ana.analyze(_single_kernel(3, 0b001, inv))
    assert rules[0] == [(FIXED, 0, (), 12345, (), 0, (), 0)] and un[0] == 0
    # a size that follows an argument which never changes is indistinguishable from a constant: T1 comes first
    inv = [([A + 16 * i, 100, m], [(A + 16 * i, 400)]) for i, m in enumerate([3, 4, 5])]
    rules, _ = ana.analyze(_single_kernel(3, 0b001, inv))
    assert rules[0] == [(FIXED, 0, (), 400, (), 0, (), 0)]


def test_strided_region_and_its_three_formulas(ana):
    # K-cache style: `batch` chunks of L*8 bytes, one every max_tokens*8 bytes
    A = 7 << 40
    inv = []
    for i, (L, mt, batch) in enumerate([(10, 512, 4), (11, 512, 4), (300, 1024, 2), (5, 64, 6), (7, 2048, 1)]):
        a = [A + 8 * i, L, mt, batch]
        inv.append((a, [(a[0] + j * mt * 8, L * 8) for j in range(batch)]))
    rules, un = ana.analyze(_single_kernel(4, 0b0001, inv))
    assert un[0] == 0
    assert rules[0] == [(STRIDED, 0, (1,), 8, (2,), 8, (3,), 1)]


def test_regions_no_argument_points_to_stay_unexplained(ana):
    A = 9 << 40
    inv = [([A + 4 * i, n], [(A + 4 * i, 2 * n), ((11 << 40) + 100 * i, 64)]) for i, n in enumerate([10, 20, 35])]
    rules, un = ana.analyze(_single_kernel(2, 0b01, inv))
    assert rules[0] == [(LINEAR, 0, (1,), 2, (), 0, (), 0)]
    assert un[0] == 3                                    # one interval per invocation
    # a pointer whose region follows no product of the arguments
    inv = [([A + 4 * i, n], [(A + 4 * i, n * n + 1)]) for i, n in enumerate([10, 20, 35])]
    rules, un = ana.analyze(_single_kernel(2, 0b01, inv))
    assert rules[0] == [] and un[0] == 3
    # an alias of a lower pointer yields no second rule
    inv = [([A + 4 * i, A + 4 * i, n], [(A + 4 * i, 8 * n)]) for i, n in enumerate([1, 2, 3])]
    rules, un = ana.analyze(_single_kernel(3, 0b011, inv))
    assert rules[0] == [(LINEAR, 0, (2,), 8, (), 0, (), 0)] and un[0] == 0
    # a 32-bit argument is never taken for a pointer even if its value matches a start address
    inv = [([1000 + i, n], [(1000 + i, 4 * n)]) for i, n in enumerate([1, 2, 3])]
    rules, un = ana.analyze(_single_kernel(2, 0b00, inv))
    assert rules[0] == [] and un[0] == 3


def test_strided_run_stops_at_an_irregular_gap_and_pointers_never_enter_products(ana):
    A = 7 << 40
    # three chunks 100 bytes apart, then a fourth of the same length 250 further on: not part of the run
    inv = [([A + 1000 * i, n], [(A + 1000 * i + j * 100, 4 * n) for j in range(3)] + [(A + 1000 * i + 450, 4 * n)])
           for i, n in enumerate([3, 5, 7])]
    rules, un = ana.analyze(_single_kernel(2, 0b01, inv))
    assert rules[0] == [(STRIDED, 0, (1,), 4, (), 100, (), 3)]
    assert un[0] == 3
    # B's address happens to equal A's size in every invocation; only the integer argument may explain it
    inv = [([A + 64 * i, 4096 * (i + 1), i + 1], [(A + 64 * i, 4096 * (i + 1)), (4096 * (i + 1), 16)]) for i in range(3)]
    rules, un = ana.analyze(_single_kernel(3, 0b011, inv))
    assert rules[0] == [(LINEAR, 0, (2,), 4096, (), 0, (), 0), (FIXED, 1, (), 16, (), 0, (), 0)] and un[0] == 0


def _first_match_by_exhaustion(values, arg_rows, candidates):
    """All (subset, coefficient) pairs that explain the values, in the search order; returns the first."""
    for size in range(0, 4):
        for S in itertools.combinations(candidates, size):
            prods = [int(np.prod([int(r[j]) for j in S], dtype=object)) if S else 1 for r in arg_rows]
            if any(p >= 1 << 64 for p in prods):
                continue
            nz = [(v, p) for v, p in zip(values, prods) if p]
            if not nz or nz[0][0] % nz[0][1]:
                continue
            c = nz[0][0] // nz[0][1]
            if c >= 1 and all(v == c * p for v, p in zip(values, prods)):
                return S, c
    return None


def test_first_match_equals_exhaustive_search(ana):
    rng = np.random.default_rng(4)
    A = 3 << 40
    for trial in range(200):
        n_int = int(rng.integers(1, 6))
        n_inv = int(rng.integers(2, 6))
        rows = [[A + 8 * i] + [int(rng.integers(0, 6)) for _ in range(n_int)] for i in range(n_inv)]
        S = tuple(sorted(rng.choice(range(1, n_int + 1), size=int(rng.integers(0, min(3, n_int) + 1)), replace=False).tolist()))
        c = int(rng.integers(1, 5))
        sizes = [c * int(np.prod([r[j] for j in S])) if S else c for r in rows]
        if any(sz == 0 for sz in sizes):                  # an empty region leaves no interval: not a valid trace
            continue
        inv = [(r, [(r[0], sz)]) for r, sz in zip(rows, sizes)]
        rules, un = ana.analyze(_single_kernel(1 + n_int, 0b1, inv))
        want = _first_match_by_exhaustion(sizes, rows, list(range(1, n_int + 1)))
        assert want is not None
        kind = FIXED if not want[0] else LINEAR
        assert rules[0] == [(kind, 0, want[0], want[1], (), 0, (), 0)], (trial, rows, sizes)


@pytest.mark.parametrize("vary", [True, False])
def test_derived_rules_reproduce_every_profiled_invocation(ana, vary):
    b = make_batch(seed=3, n_kernels=120, n_inv=12, vary=vary)
    rules, un = ana.analyze(b)
    for k in range(b.n_kernels):
        assert un[k] == b.n_other[k] * b.n_inv, k
        assert len(rules[k]) == len(b.hidden[k])
        for i in range(b.n_inv):
            got = sorted(iv for r in rules[k] for iv in _predict(r, b.args[k, i]))
            want = sorted((int(s), int(l)) for s, l in b.iv[k, i, :b.n_iv[k, i]])
            other = [w for w in want if (w[0] >> 40) == 60]
            assert got == [w for w in want if w not in other], (k, i)
        if vary:                                          # identifiable: the hidden model itself comes back
            for r, h in zip(rules[k], b.hidden[k]):
                if h.kind == STRIDED:
                    continue                              # a count that is always 1 in the sample legitimately degenerates
                assert r[0] == h.kind and r[1] == h.base_arg and r[2] == h.size_args and r[3] == h.size_coeff, (k, r, h)


def test_buffers_that_touch_or_overlap_are_still_told_apart(ana):
    # A and B are neighbours in memory (B begins where A ends); C overlaps the tail of B.  One interval per
    # memory instruction, so each pointer still begins an interval and gets its own rule.
    A = 9 << 40
    inv = []
    for n in (3, 8, 5, 13):
        B = A + 4 * n
        C = B + 8
        inv.append(([A, B, C, n], [(A, 4 * n), (B, 64), (C, 16 * n)]))
    rules, un = ana.analyze(_single_kernel(4, 0b0111, inv))
    assert rules[0] == [(LINEAR, 0, (3,), 4, (), 0, (), 0), (FIXED, 1, (), 64, (), 0, (), 0), (LINEAR, 2, (3,), 16, (), 0, (), 0)]
    assert un[0] == 0


def test_a_base_pointer_starts_a_region_in_every_invocation(ana):
    """Sec. 5.2: a base pointer is a 64-bit argument that appears as the beginning address of a region.  A 64-bit
    integer that happens to equal some region's start in one invocation only is not one: it yields no rule of its
    own and stays available as a factor of the size."""
    A, B = 9 << 40, 11 << 40
    inv = []
    for i, n in enumerate([B // 8, 1000, 4096, 77]):            # invocation 0: 8 * n == B, and n == the start of a region
        a = [A + 32 * i, n]
        rows = [(a[0], 8 * n)]
        if i == 0:
            rows.append((n, 64))                                 # some other buffer happens to begin at address n
        inv.append((a, rows))
    rules, un = ana.analyze(_single_kernel(2, 0b11, inv))
    assert rules[0] == [(LINEAR, 0, (1,), 8, (), 0, (), 0)]
    assert un[0] == 1
