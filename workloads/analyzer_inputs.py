"""Seeded synthetic profiler output for the offline memory analyzer (Sec. 5.2 of the paper: the
profiler records, for every invocation of a kernel, its launch arguments and the addresses it
touched).  A kernel is drawn from a hidden model (which argument is a pointer, how each region's
extent follows from the other arguments) and its invocations are played forward into touched byte
intervals; the analyzer sees only arguments and intervals and has to find the model again."""
from dataclasses import dataclass
from typing import List

import numpy as np

MAX_ARGS = 12
FIXED, LINEAR, STRIDED, OTHER = 1, 2, 3, 0


@dataclass
class HiddenRule:
    kind: int
    base_arg: int
    size_args: tuple = ()
    size_coeff: int = 0
    stride_args: tuple = ()
    stride_coeff: int = 0
    count_args: tuple = ()
    count_coeff: int = 0


@dataclass
class AnalyzerBatch:
    n_kernels: int
    n_inv: int
    max_iv: int
    n_args: np.ndarray      # int32  [K]
    ptr_mask: np.ndarray    # uint32 [K]   bit a: argument a is a 64-bit integer
    args: np.ndarray        # uint64 [K, n_inv, MAX_ARGS]
    iv: np.ndarray          # uint64 [K, n_inv, max_iv, 2]  (start, length), sorted by start
    n_iv: np.ndarray        # uint32 [K, n_inv]
    hidden: List[List[HiddenRule]]
    n_other: np.ndarray     # intervals per invocation that no argument explains


def _prod(vals):
    out = 1
    for v in vals:
        out *= int(v)
    return out


def make_batch(seed=0, n_kernels=64, n_inv=16, max_iv=48, vary=True) -> AnalyzerBatch:
    """vary=True: every size-like argument changes between invocations (the hidden model is
    identifiable); vary=False: some stay constant, as in real applications, so a simpler rule than the
    hidden one can explain the trace."""
    rng = np.random.default_rng([seed, 11])
    n_args = np.zeros(n_kernels, np.int32)
    ptr_mask = np.zeros(n_kernels, np.uint32)
    args = np.zeros((n_kernels, n_inv, MAX_ARGS), np.uint64)
    iv = np.zeros((n_kernels, n_inv, max_iv, 2), np.uint64)
    n_iv = np.zeros((n_kernels, n_inv), np.uint32)
    n_other = np.zeros(n_kernels, np.uint32)
    hidden = []
    for k in range(n_kernels):
        n_rules = int(rng.integers(1, 5))
        n_ptr = n_rules + int(rng.integers(0, 2))                 # sometimes a pointer nothing is read through
        n_int = int(rng.integers(3, MAX_ARGS - n_ptr + 1))
        na = n_ptr + n_int
        n_args[k] = na
        ints = list(range(n_ptr, na))
        mask = (1 << n_ptr) - 1
        for a in ints:                                            # some sizes are passed as 64-bit integers
            if rng.random() < 0.3:
                mask |= 1 << a
        ptr_mask[k] = mask
        rules, limit = [], {a: 200 for a in ints}                 # limit: largest value an argument may take
        for r in range(n_rules):
            u = rng.random()
            kind = FIXED if u < 0.5 else (LINEAR if u < 0.85 else STRIDED)
            if kind == FIXED:
                rules.append(HiddenRule(FIXED, r, (), int(rng.integers(1, 1 << 20))))
            elif kind == LINEAR:
                m = int(rng.integers(1, 3))
                S = tuple(sorted(rng.choice(ints, size=m, replace=False).tolist()))
                rules.append(HiddenRule(LINEAR, r, S, int(rng.choice([1, 2, 4, 8, 12]))))
            else:
                s_, t_, c_ = (int(x) for x in rng.choice(ints, size=3, replace=False))
                limit[s_] = min(limit[s_], 100); limit[t_] = min(limit[t_], 8); limit[c_] = min(limit[c_], 5)
                # chunk <= 16 * 100 bytes, stride >= 4096 bytes: chunks never touch
                rules.append(HiddenRule(STRIDED, r, (s_,), int(rng.choice([2, 4, 16])), (t_,), int(rng.choice([4096, 8192])),
                                        (c_,), 1))
        hidden.append(rules)
        has_other = rng.random() < 0.2
        n_other[k] = 1 if has_other else 0
        constant = {a: (not vary) and rng.random() < 0.5 for a in ints}
        const_val = {a: int(rng.integers(1, limit[a] + 1)) for a in ints}
        for i in range(n_inv):
            for a in ints:
                args[k, i, a] = const_val[a] if constant[a] else int(rng.integers(1, limit[a] + 1))
            rows = []
            for r, q in enumerate(rules):
                base = ((r + 1) << 40) + int(rng.integers(0, 1 << 30)) * 4     # every region in its own address window
                args[k, i, q.base_arg] = base
                a_i = [int(x) for x in args[k, i]]
                if q.kind == FIXED:
                    rows.append((base, q.size_coeff))
                elif q.kind == LINEAR:
                    rows.append((base, q.size_coeff * _prod(a_i[s] for s in q.size_args)))
                else:
                    chunk = q.size_coeff * a_i[q.size_args[0]]
                    stride = q.stride_coeff * a_i[q.stride_args[0]]
                    for j in range(q.count_coeff * a_i[q.count_args[0]]):
                        rows.append((base + j * stride, chunk))
            for p in range(n_rules, n_ptr):                       # unused pointers point somewhere untouched
                args[k, i, p] = (50 << 40) + int(rng.integers(0, 1 << 30)) * 4
            if has_other:                                         # data reached through a pointer held in memory
                rows.append(((60 << 40) + int(rng.integers(0, 1 << 30)) * 4, int(rng.integers(1, 4096))))
            rows.sort()
            assert len(rows) <= max_iv
            for m in range(1, len(rows)):
                assert rows[m - 1][0] + rows[m - 1][1] < rows[m][0], "intervals must not touch"
            n_iv[k, i] = len(rows)
            for m, (st, ln) in enumerate(rows):
                iv[k, i, m] = (st, ln)
    return AnalyzerBatch(n_kernels, n_inv, max_iv, n_args, ptr_mask, args, iv, n_iv, hidden, n_other)


def make_adversarial_batch(seed=0, n_kernels=64, n_inv=8, max_iv=32) -> AnalyzerBatch:
    """Profiler output full of coincidences: tiny integer arguments, some duplicated or constant (many
    argument subsets explain the same extent; the order of the search decides), zero-valued arguments,
    pointers into the middle of a strided run, pointers that coincide in some or all invocations,
    neighbouring groups of chunks that line up into one longer run, and 64-bit integers large enough
    to overflow a product."""
    rng = np.random.default_rng([seed, 13])
    n_args = np.zeros(n_kernels, np.int32)
    ptr_mask = np.zeros(n_kernels, np.uint32)
    args = np.zeros((n_kernels, n_inv, MAX_ARGS), np.uint64)
    iv = np.zeros((n_kernels, n_inv, max_iv, 2), np.uint64)
    n_iv = np.zeros((n_kernels, n_inv), np.uint32)
    step = 4096
    for k in range(n_kernels):
        n_groups = int(rng.integers(1, 4))
        n_ptr = int(rng.integers(1, 5))
        n_int = int(rng.integers(1, MAX_ARGS - n_ptr + 1))
        na = n_ptr + n_int
        n_args[k] = na
        order = rng.permutation(na)                               # pointers and integers interleaved
        ptr_args, int_args = sorted(order[:n_ptr].tolist()), sorted(order[n_ptr:].tolist())
        mask = sum(1 << a for a in ptr_args)
        for a in int_args:
            if rng.random() < 0.4:
                mask |= 1 << a
        ptr_mask[k] = mask
        int_role = {a: int(rng.choice([0, 0, 0, 1, 2, 3])) for a in int_args}   # 0 tiny, 1 constant, 2 copy, 3 huge
        sub = lambda hi: tuple(sorted(rng.choice(int_args, size=min(len(int_args), int(rng.integers(0, hi))),
                                                  replace=False).tolist()))
        groups = [dict(len_c=int(rng.choice([4, 8, 16])), len_s=sub(4), cnt_s=sub(3), str_s=sub(2),
                       glue=rng.random() < 0.3) for _ in range(n_groups)]
        ptr_role = {a: (int(rng.integers(0, n_groups)), int(rng.choice([0, 0, 0, 1])), rng.random() < 0.15)
                    for a in ptr_args}                            # (group, chunk pointed at, sometimes elsewhere)
        const_val = {a: int(rng.integers(1, 4)) for a in int_args}
        for i in range(n_inv):
            for a in int_args:
                r = int_role[a]
                if r == 1:
                    v = const_val[a]
                elif r == 2 and a != int_args[0]:
                    v = int(args[k, i, int_args[0]])
                elif r == 3:
                    v = int(rng.integers(1 << 40, 1 << 62))
                else:
                    v = int(rng.integers(0, 4)) if rng.random() < 0.1 else int(rng.integers(1, 4))
                args[k, i, a] = v
            val = lambda S: _prod(min(int(args[k, i, a]), 3) for a in S)
            rows, starts, cursor = [], [], (1 << 40) + int(rng.integers(0, 1 << 20)) * step
            for g in groups:
                ln = max(1, g["len_c"] * val(g["len_s"]))
                cnt = max(1, val(g["cnt_s"]))
                stride = step * max(1, val(g["str_s"]))
                if not (g["glue"] and rows):                      # glued: continues the previous group's grid
                    cursor += step * int(rng.integers(2, 6))
                first = len(rows)
                for j in range(cnt):
                    if len(rows) < max_iv:
                        rows.append((cursor + j * stride, ln))
                starts.append((first, len(rows)))
                cursor = rows[-1][0] + stride
            for a in ptr_args:
                g, chunk, stray = ptr_role[a]
                lo, hi = starts[g]
                m = min(lo + chunk, max(hi - 1, lo)) if hi > lo else 0
                if stray and rng.random() < 0.5:
                    m = int(rng.integers(0, len(rows)))
                args[k, i, a] = rows[min(m, len(rows) - 1)][0]
            n_iv[k, i] = len(rows)
            for m, (st, ln) in enumerate(rows):
                iv[k, i, m] = (st, ln)
    return AnalyzerBatch(n_kernels, n_inv, max_iv, n_args, ptr_mask, args, iv, n_iv, [[] for _ in range(n_kernels)],
                         np.zeros(n_kernels, np.uint32))
