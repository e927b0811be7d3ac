"""Degraded predictors for the ablations of the paper (Sec. 5.1 "Naive solution: allocation-granularity
prediction", Sec. 5.2 on false negatives, Sec. 7 Fig. "eval-naive").  They rewrite a schedule's templates and
launch arguments only: what the planner is *told* a launch will touch.  No page set is computed here."""
import dataclasses

import numpy as np

from .trace import MAX_ARGS, RULE_LINEAR, RULE_LIST, Rule, Trace, CommandBuilder


def allocation_granularity(trace: Trace) -> Trace:
    """The same launches as predicted by the naive scheme: every pointer argument that falls inside a buffer the
    task allocated is taken to touch the whole buffer.  Each launch gets a template of one LINEAR rule per
    pointer, (base = buffer start, size = 1 x buffer bytes), with starts and sizes as its arguments."""
    assert trace.allocations is not None and len(trace.allocations), "the schedule does not record its allocations"
    starts = trace.allocations[:, 0].astype(np.int64)
    sizes = trace.allocations[:, 1].astype(np.int64)
    assert (np.diff(starts) > 0).all()
    kernels, tasks, naive_of = [], [], {}
    for cmds in trace.tasks:
        b = CommandBuilder()
        for i in range(len(cmds)):
            rules = trace.kernels[int(cmds.kernel_id[i])]
            assert all(r.kind != RULE_LIST for r in rules), "id lists carry no pointer to look up"
            assert 2 * len(rules) <= MAX_ARGS
            args = []
            for r in rules:
                ptr = int(cmds.args[i, r.base_arg])
                a = int(np.searchsorted(starts, ptr, side="right")) - 1
                assert a >= 0 and ptr < starts[a] + sizes[a], "pointer outside every allocation"
                args.append(a)
            n = len(rules)
            if n not in naive_of:
                naive_of[n] = len(kernels)
                kernels.append([Rule(RULE_LINEAR, j, (n + j,), 1) for j in range(n)])
            b.add(naive_of[n], [int(starts[a]) for a in args] + [int(sizes[a]) for a in args],
                  latency=int(cmds.latency[i]))
        tasks.append(b.build())
    return dataclasses.replace(trace, name=trace.name + "+allocation-granularity", kernels=kernels, tasks=tasks)


def drop_rules(trace: Trace, rate: float, seed: int = 0) -> Trace:
    """False negatives: each (launch, rule) prediction is lost with probability `rate` (the launch is then
    predicted through a template without that rule).  The launches themselves are unchanged."""
    rng = np.random.default_rng([seed, 17])
    kernels = [list(k) for k in trace.kernels]
    variant = {}
    tasks = []
    for cmds in trace.tasks:
        kid = cmds.kernel_id.copy()
        for i in range(len(cmds)):
            k = int(cmds.kernel_id[i])
            keep = tuple(bool(rng.random() >= rate) for _ in trace.kernels[k])
            if all(keep):
                continue
            if (k, keep) not in variant:
                variant[(k, keep)] = len(kernels)
                kernels.append([r for r, kp in zip(trace.kernels[k], keep) if kp])
            kid[i] = variant[(k, keep)]
        tasks.append(dataclasses.replace(cmds, kernel_id=kid))
    return dataclasses.replace(trace, name=f"{trace.name}+drop{rate}", kernels=kernels, tasks=tasks)
