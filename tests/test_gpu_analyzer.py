"""HIP memory analyzer (msched_analyze, Sec. 5.2 "Memory analyzer" of the paper) against the plain-C
oracle: rule for rule, field for field, on seeded profiler output."""
import numpy as np
import pytest

from workloads.analyzer_inputs import make_batch, make_adversarial_batch, AnalyzerBatch, MAX_ARGS

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def oracle_analyzer():
    from oracle import analyzer
    analyzer.build()
    return analyzer


def hip_analyze(batch: AnalyzerBatch):
    import torch
    import paper_2512_24637_amd as M
    dev = torch.device("cuda:0")
    up = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a).view(dt)).to(dev)
    K = batch.n_kernels
    n_args, mask = up(batch.n_args, np.int32), up(batch.ptr_mask, np.int32)
    args, iv, n_iv = up(batch.args, np.int64), up(batch.iv, np.int64), up(batch.n_iv, np.int32)
    rules = torch.zeros((max(K, 1), 8, 48), dtype=torch.uint8, device=dev)
    n_rules = torch.full((max(K, 1),), -1, dtype=torch.int32, device=dev)
    unexplained = torch.full((max(K, 1),), -1, dtype=torch.int32, device=dev)
    M.analyze(K, batch.n_inv, batch.max_iv, n_args.data_ptr(), mask.data_ptr(), args.data_ptr(), iv.data_ptr(),
              n_iv.data_ptr(), rules.data_ptr(), n_rules.data_ptr(), unexplained.data_ptr(),
              torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    nr = n_rules.cpu().numpy()[:K]
    return M.rules_from_bytes(rules.cpu().numpy()[:K], nr), unexplained.cpu().numpy()[:K].astype(np.uint32)


def assert_same(batch, oracle_analyzer):
    want, want_un = oracle_analyzer.analyze(batch)
    got, got_un = hip_analyze(batch)
    for k in range(batch.n_kernels):
        assert got[k] == want[k], f"kernel {k}: {got[k]} != {want[k]}"
    assert np.array_equal(got_un, want_un)
    return want


@pytest.mark.parametrize("vary", [True, False])
@pytest.mark.parametrize("seed", [0, 1])
def test_model_batches(oracle_analyzer, seed, vary):
    want = assert_same(make_batch(seed, n_kernels=192, n_inv=16, max_iv=48, vary=vary), oracle_analyzer)
    assert sum(len(r) for r in want) > 192


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_adversarial_batches(oracle_analyzer, seed):
    want = assert_same(make_adversarial_batch(seed, n_kernels=384, n_inv=8, max_iv=32), oracle_analyzer)
    kinds = {r[0] for rs in want for r in rs}
    assert kinds == {1, 2, 3}


@pytest.mark.parametrize("n_inv", [63, 64, 65, 130])
def test_invocations_around_one_per_lane(oracle_analyzer, n_inv):
    """A lane keeps the first eight intervals of one invocation in registers and follows runs through them with fixed
    indices; invocations beyond the first 64, and intervals beyond the eighth, are read from memory.  Batches of the
    shape bench.py times (64 invocations, runs of up to 13 chunks) and one invocation more or less than the lanes,
    model and adversarial."""
    assert_same(make_batch(7, n_kernels=128, n_inv=n_inv, max_iv=48, vary=True), oracle_analyzer)
    assert_same(make_batch(8, n_kernels=128, n_inv=n_inv, max_iv=48, vary=False), oracle_analyzer)
    assert_same(make_adversarial_batch(9, n_kernels=128, n_inv=n_inv, max_iv=32), oracle_analyzer)


def test_shapes_at_the_limits(oracle_analyzer):
    # the most invocations one call takes, more than one pass of the workgroup over them
    assert_same(make_batch(3, n_kernels=6, n_inv=512, max_iv=48, vary=True), oracle_analyzer)
    assert_same(make_adversarial_batch(4, n_kernels=16, n_inv=300, max_iv=64), oracle_analyzer)
    # one invocation: every extent is "invariant"
    assert_same(make_batch(5, n_kernels=32, n_inv=1, max_iv=48, vary=True), oracle_analyzer)
    assert_same(make_adversarial_batch(6, n_kernels=64, n_inv=2, max_iv=32), oracle_analyzer)


def test_kernel_without_arguments_or_intervals(oracle_analyzer):
    K, n_inv, max_iv = 3, 4, 4
    b = AnalyzerBatch(K, n_inv, max_iv, np.array([0, 2, 1], np.int32), np.array([0, 3, 1], np.uint32),
                      np.zeros((K, n_inv, MAX_ARGS), np.uint64), np.zeros((K, n_inv, max_iv, 2), np.uint64),
                      np.zeros((K, n_inv), np.uint32), [[]] * K, np.zeros(K, np.uint32))
    b.args[2, :, 0] = 4096                       # a pointer, but the kernel touched nothing
    b.iv[1, :, 0] = (0, 64); b.n_iv[1] = 1       # both arguments of kernel 1 are 0 = the interval's start: aliases
    want = assert_same(b, oracle_analyzer)
    assert want[0] == [] and want[2] == [] and len(want[1]) == 1


def test_argument_errors():
    import torch
    import paper_2512_24637_amd as M
    d = torch.zeros(1024, dtype=torch.int64, device="cuda:0").data_ptr()
    M.analyze(0, 4, 4, d, d, d, d, d, d, d, d)                       # empty batch: nothing to do
    for n_inv, max_iv in [(0, 4), (513, 4), (4, 0), (4, 65536)]:
        with pytest.raises(M.MSchedError) as e:
            M.analyze(1, n_inv, max_iv, d, d, d, d, d, d, d, d)
        assert e.value.code == -1
    with pytest.raises(M.MSchedError):
        M.analyze(1, 4, 4, d, d, 0, d, d, d, d, d)


# ---- closing the loop: templates derived by the analyzer drive the planner like the hand-written ones ----

def _ranges_of(rules, args):
    """Byte ranges a launch touches under a kernel template (forward evaluation of the rule definition)."""
    out = []
    prod = lambda idx: int(np.prod([int(args[j]) for j in idx], dtype=object)) if len(idx) else 1
    for r in rules:
        kind, base_arg, s_idx, s_c, t_idx, t_c, c_idx, c_c = r
        base, size = int(args[base_arg]), s_c * prod(s_idx)
        if kind in (1, 2):
            out.append((base, size))
        else:
            out += [(base + j * t_c * prod(t_idx), size) for j in range(c_c * prod(c_idx))]
    return [(a, b) for a, b in out if b > 0]


def _merged(ranges):
    """What the profiler reports: one interval per region a memory instruction covers; regions that begin at
    the same address become one.  Regions of different buffers stay apart even where they touch or overlap."""
    out = []
    for a, b in sorted(ranges):
        if out and a == out[-1][0]:
            out[-1] = (a, max(out[-1][1], b))
        else:
            out.append((a, b))
    return out


def _pages(ranges, shift):
    s = set()
    for a, b in ranges:
        s.update(range(a >> shift, ((a + b - 1) >> shift) + 1))
    return s


def _as_tuple(r):
    return (r.kind, r.base_arg, tuple(r.size_args), r.size_coeff, tuple(r.stride_args), r.stride_coeff,
            tuple(r.count_args), r.count_coeff)


@pytest.mark.parametrize("config,kw", [(1, {}), (3, dict(scale=16, n_launches=480)), (4, dict(page_shift=16, n_launches=512))])
def test_derived_templates_drive_the_same_plans(oracle_mod, oracle_analyzer, config, kw):
    import dataclasses
    from workloads import make_trace, run_schedule
    from workloads.trace import Rule
    from gpu_common import GpuSide, make_oracle, assert_same_plan
    trace = make_trace(config, **kw)
    hand = [[_as_tuple(r) for r in rules] for rules in trace.kernels]
    # "profile" every kernel: its launches' arguments and the intervals its template touches
    launches = {k: [] for k in range(len(hand))}
    for cmds in trace.tasks:
        for i in range(len(cmds)):
            launches[int(cmds.kernel_id[i])].append((int(cmds.n_args[i]), cmds.args[i]))
    n_inv = min(512, max(len(v) for v in launches.values()))
    prof = {k: [v[j * len(v) // n_inv] for j in range(n_inv)] for k, v in launches.items() if v}
    rows = {k: [_merged(_ranges_of(hand[k], a)) for _, a in v] for k, v in prof.items()}
    K, max_iv = len(hand), max(len(r) for v in rows.values() for r in v)
    b = AnalyzerBatch(K, n_inv, max_iv, np.zeros(K, np.int32), np.zeros(K, np.uint32),
                      np.zeros((K, n_inv, MAX_ARGS), np.uint64), np.zeros((K, n_inv, max_iv, 2), np.uint64),
                      np.zeros((K, n_inv), np.uint32), [[]] * K, np.zeros(K, np.uint32))
    for k, v in prof.items():
        b.n_args[k] = v[0][0]
        b.ptr_mask[k] = (1 << v[0][0]) - 1                  # nothing says which arguments are pointers
        for i, (_, a) in enumerate(v):
            b.args[k, i] = a
            b.n_iv[k, i] = len(rows[k][i])
            for m, iv in enumerate(rows[k][i]):
                b.iv[k, i, m] = iv
    derived = assert_same(b, oracle_analyzer)
    # the derived templates must predict the pages of every launch, profiled or not
    for k, v in launches.items():
        for na, a in v:
            assert _pages(_ranges_of(derived[k], a), trace.page_shift) == _pages(_ranges_of(hand[k], a), trace.page_shift), (k, a[:na])
    # and the planner, fed with them, must decide exactly what the oracle decides from the hand-written ones
    t2 = dataclasses.replace(trace, kernels=[[Rule(*r) for r in rs] for rs in derived])
    g = GpuSide(t2)
    o = make_oracle(oracle_mod, trace, with_bytes=False)
    try:
        n = 0
        for ro, rg in zip(run_schedule(trace, o, max_plans=24), run_schedule(t2, g.ms, max_plans=24)):
            assert_same_plan(ro.plan, rg.plan, (trace.name, "plan", ro.index))
            pto, foo = o.state()
            ptg, fog = g.ms.state()
            assert np.array_equal(pto, ptg) and np.array_equal(foo, fog)
            n += 1
        assert n > 3
    finally:
        g.close()
        o.close()
