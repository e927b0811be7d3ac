"""Pins for the oracle's template expander (Sec. 5.2 of the paper: T1/T2/T3 templates,
page alignment).  The expected values come from definitions written out here
independently: byte marking on a small address space, and the paper's two
worked kernels (vector_add, matrix_mul)."""
import numpy as np
import pytest

from workloads import Rule, RULE_FIXED, RULE_LINEAR, RULE_STRIDED, RULE_LIST


def _mk(oracle_mod, page_shift=6, V=64, F=8, slot=None, n_slots=0):
    return oracle_mod.Oracle(page_shift, V, F, host_slot=slot, n_slots=n_slots)


def _pages_by_byte_marking(ranges, page_shift, n_bytes):
    """Definition: a page is in the set iff at least one byte of some range lies in it."""
    mark = np.zeros(n_bytes, bool)
    for a, ln in ranges:
        mark[a:a + ln] = True
    return np.unique(np.nonzero(mark)[0] >> page_shift).astype(np.uint32)


def test_random_rules_match_byte_marking(oracle_mod):
    rng = np.random.default_rng(7)
    shift, V = 6, 64
    n_bytes = V << shift
    for trial in range(300):
        o = _mk(oracle_mod, shift, V)
        t = o.task_create()
        n_rules = int(rng.integers(1, 5))
        rules, args, ranges = [], [], []
        for r in range(n_rules):
            if len(args) > 8:
                break
            kind = int(rng.choice([RULE_FIXED, RULE_LINEAR, RULE_STRIDED]))
            base = int(rng.integers(0, n_bytes - 600))
            base_idx = len(args)
            args.append(base)
            if kind == RULE_FIXED:
                size = int(rng.integers(0, 300))
                rules.append(Rule(RULE_FIXED, base_idx, (), size))
                ranges.append((base, size))
            elif kind == RULE_LINEAR:
                a, b, c = int(rng.integers(0, 9)), int(rng.integers(1, 7)), int(rng.integers(1, 6))
                i0 = len(args)
                args.extend([a, b])
                rules.append(Rule(RULE_LINEAR, base_idx, (i0, i0 + 1), c))
                ranges.append((base, a * b * c))
            else:
                chunk_n, stride_n, count = int(rng.integers(0, 40)), int(rng.integers(1, 60)), int(rng.integers(0, 6))
                i0 = len(args)
                args.extend([chunk_n, stride_n, count])
                rules.append(Rule(RULE_STRIDED, base_idx, (i0,), 2, (i0 + 1,), 3, (i0 + 2,), 1))
                for j in range(count):
                    ranges.append((base + j * stride_n * 3, chunk_n * 2))
        kid = o.kernel_register(rules)
        if any(a + ln > n_bytes for a, ln in ranges):
            with pytest.raises(oracle_mod.OracleError) as e:
                o.launch_enqueue(t, kid, args, len(args))
            assert e.value.name == "E_RANGE"
            continue
        o.launch_enqueue(t, kid, args, len(args))
        got = o.command_pages(t, 0)
        want = _pages_by_byte_marking(ranges, shift, n_bytes)
        assert np.array_equal(got, want), (trial, rules, args)


def test_paper_vector_add_and_matrix_mul(oracle_mod):
    """vector_add(A,B,C,N): all three extents scale with N; matrix_mul(A,B,C,M,N,K):
    extents scale with M*K, K*N and M*N (Sec. 5.2, T2 example)."""
    shift, V = 12, 4096
    P = 1 << shift
    o = _mk(oracle_mod, shift, V)
    t = o.task_create()
    vadd = o.kernel_register([Rule(RULE_LINEAR, i, (3,), 4) for i in range(3)])
    mm = o.kernel_register([Rule(RULE_LINEAR, 0, (3, 5), 4), Rule(RULE_LINEAR, 1, (5, 4), 4),
                            Rule(RULE_LINEAR, 2, (3, 4), 4)])
    A, B, Cc = 100 * P, 1000 * P, 2000 * P
    N = 5000                                   # 20000 bytes -> 5 pages each
    o.launch_enqueue(t, vadd, [A, B, Cc, N], 4)
    want = np.concatenate([np.arange(100, 105), np.arange(1000, 1005), np.arange(2000, 2005)])
    assert np.array_equal(o.command_pages(t, 0), want)
    o.launch_enqueue(t, vadd, [A, B, Cc, 2 * N], 4)     # doubling N doubles every extent
    assert o.command_pages(t, 1).size == 3 * 10 - 0 and o.command_pages(t, 1)[9] == 109
    M, N2, K = 64, 48, 80                      # A: 64*80*4 = 20480 B = 5 pages; B: 80*48*4 = 15360 B = 3.75 -> 4; C: 64*48*4 = 12288 B = 3
    o.launch_enqueue(t, mm, [A, B, Cc, M, N2, K], 6)
    want = np.concatenate([np.arange(100, 105), np.arange(1000, 1004), np.arange(2000, 2003)])
    assert np.array_equal(o.command_pages(t, 2), want)


def test_alignment_is_outward_and_empty_ranges_touch_nothing(oracle_mod):
    shift, V = 8, 32
    P = 1 << shift
    o = _mk(oracle_mod, shift, V)
    t = o.task_create()
    k = o.kernel_register([Rule(RULE_LINEAR, 0, (1,), 1)])
    cases = [
        (3 * P, 0, []),                    # zero bytes: nothing
        (3 * P, 1, [3]),                   # one byte at a page start
        (4 * P - 1, 1, [3]),               # last byte of a page
        (4 * P - 1, 2, [3, 4]),            # straddles a boundary
        (3 * P, P, [3]),                   # exactly one page
        (3 * P, P + 1, [3, 4]),            # one byte over
        (3 * P + 5, 2 * P, [3, 4, 5]),     # ragged both ends
    ]
    for i, (base, n, want) in enumerate(cases):
        o.launch_enqueue(t, k, [base, n], 2)
        assert o.command_pages(t, i).tolist() == want


def test_strided_with_chunk_equal_to_stride_is_one_linear_range(oracle_mod):
    shift, V = 8, 256
    o = _mk(oracle_mod, shift, V)
    t = o.task_create()
    ks = o.kernel_register([Rule(RULE_STRIDED, 0, (1,), 8, (1,), 8, (2,), 1)])
    kl = o.kernel_register([Rule(RULE_LINEAR, 0, (1, 2), 8)])
    rng = np.random.default_rng(3)
    for i in range(50):
        base, n, cnt = int(rng.integers(0, 4000)), int(rng.integers(1, 300)), int(rng.integers(1, 20))
        o.launch_enqueue(t, ks, [base, n, cnt], 3)
        o.launch_enqueue(t, kl, [base, n, cnt], 3)
        assert np.array_equal(o.command_pages(t, 2 * i), o.command_pages(t, 2 * i + 1))


def test_list_rule_dedupes_and_sorts(oracle_mod):
    o = _mk(oracle_mod, 8, 100)
    t = o.task_create()
    k = o.kernel_register([Rule(RULE_LIST), Rule(RULE_FIXED, 0, (), 256)])
    o.launch_enqueue(t, k, [7 * 256], 1, ids=np.array([9, 3, 9, 99, 3, 7], np.uint32))
    assert o.command_pages(t, 0).tolist() == [3, 7, 9, 99]
    with pytest.raises(oracle_mod.OracleError) as e:
        o.launch_enqueue(t, k, [0], 1, ids=np.array([100], np.uint32))
    assert e.value.name == "E_RANGE"


def test_errors(oracle_mod):
    o = _mk(oracle_mod, 8, 64)
    t = o.task_create()
    k = o.kernel_register([Rule(RULE_LINEAR, 0, (1, 2), 1 << 40)])
    with pytest.raises(oracle_mod.OracleError) as e:     # product overflows 64 bits
        o.launch_enqueue(t, k, [0, 1 << 20, 1 << 20], 3)
    assert e.value.name == "E_OVERFLOW"
    with pytest.raises(oracle_mod.OracleError) as e:     # rule names an argument that was not passed
        o.launch_enqueue(t, k, [0, 1], 2)
    assert e.value.name == "E_RANGE"
    k2 = o.kernel_register([Rule(RULE_LINEAR, 0, (1,), 1)])
    with pytest.raises(oracle_mod.OracleError) as e:     # base + size wraps
        o.launch_enqueue(t, k2, [(1 << 64) - 10, 100], 2)
    assert e.value.name == "E_OVERFLOW"
    with pytest.raises(oracle_mod.OracleError) as e:     # past the end of the page table
        o.launch_enqueue(t, k2, [63 * 256, 257], 2)
    assert e.value.name == "E_RANGE"
    with pytest.raises(oracle_mod.OracleError) as e:
        o.launch_enqueue(t, 99, [0], 1)
    assert e.value.name == "E_INVAL"
    # pages without a backing slot may not be used
    slot = np.full(64, 0xFFFFFFFF, np.uint32)
    slot[:8] = np.arange(8)
    o2 = _mk(oracle_mod, 8, 64, slot=slot, n_slots=8)
    t2 = o2.task_create()
    k3 = o2.kernel_register([Rule(RULE_LINEAR, 0, (1,), 1)])
    o2.launch_enqueue(t2, k3, [0, 8 * 256], 2)
    with pytest.raises(oracle_mod.OracleError) as e:
        o2.launch_enqueue(t2, k3, [0, 8 * 256 + 1], 2)
    assert e.value.name == "E_RANGE"
