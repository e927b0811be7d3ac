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
