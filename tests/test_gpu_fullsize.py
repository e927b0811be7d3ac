"""The five benchmark configurations at their full sizes, in the launch configuration bench.py
times: lists, page table and frame owners bit-exact against the oracle after every switch, bytes
checked on a seeded sample of pages whose contents are tracked one by one (needs an MI355X)."""
import pytest

from workloads import make_trace
from gpu_common import lockstep_sampled

pytestmark = pytest.mark.gpu


def _log(msg):
    print(msg, flush=True)


def test_c2_stencil_full_size(oracle_mod):
    assert lockstep_sampled(oracle_mod, make_trace(2), n_sample=512, check_every=5, log=_log) == 80


def test_c3_training_full_size_all_20_iterations(oracle_mod):
    trace = make_trace(3)                          # full layer sizes and pool, all 20 iterations of both tasks
    assert sum(len(t) for t in trace.tasks) == 2 * 20 * 96
    assert lockstep_sampled(oracle_mod, trace, n_sample=8192, check_every=4, log=_log) >= 40


def test_c4_decode_full_size_all_256_steps(oracle_mod):
    trace = make_trace(4)                          # full model and pool, all 256 decode steps of both tasks:
    assert sum(len(t) for t in trace.tasks) == 2 * 256 * 64      # the cached sequence grows from 385 to 640 tokens
    assert lockstep_sampled(oracle_mod, trace, n_sample=1024, check_every=8, log=_log) == 128


def test_c5_planning_stress_full_size_all_5000_launches(oracle_mod):
    trace = make_trace(5)                          # full page counts, all 625 launches of each of the 8 tasks
    assert sum(len(t) for t in trace.tasks) == 5000
    assert lockstep_sampled(oracle_mod, trace, n_sample=16384, check_every=10, log=_log) == 104      # 12.5 timeslices per task


def test_c6_priority_colocation_full_size_first_requests(oracle_mod):
    from workloads import run_priority_schedule
    from gpu_common import lockstep
    trace = make_trace(6, requests=3, be_iterations=2)           # full layer sizes and pool (13.5 GiB); 3 requests
    n = lockstep(oracle_mod, trace, with_bytes=False, log=_log,
                 driver=lambda tr, impl, max_plans: run_priority_schedule(tr, impl, max_plans))
    assert n >= 5
