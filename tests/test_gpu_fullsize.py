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


def test_c3_training_full_size_first_switches(oracle_mod):
    trace = make_trace(3, iterations=3)            # full layer sizes and pool; 3 of the 20 iterations
    assert lockstep_sampled(oracle_mod, trace, n_sample=8192, check_every=2, log=_log) >= 6


def test_c4_decode_full_size_first_switches(oracle_mod):
    trace = make_trace(4, steps=24)                # full model and pool; 24 of the 256 decode steps
    assert lockstep_sampled(oracle_mod, trace, n_sample=1024, check_every=3, log=_log) >= 12


def test_c5_planning_stress_full_size_first_switches(oracle_mod):
    trace = make_trace(5, n_launches=100)          # full page counts; 100 of the 625 launches per task
    assert lockstep_sampled(oracle_mod, trace, n_sample=16384, check_every=4, log=_log) >= 16


def test_c6_priority_colocation_full_size_first_requests(oracle_mod):
    from workloads import run_priority_schedule
    from gpu_common import lockstep
    trace = make_trace(6, requests=3, be_iterations=2)           # full layer sizes and pool (13.5 GiB); 3 requests
    n = lockstep(oracle_mod, trace, with_bytes=False, log=_log,
                 driver=lambda tr, impl, max_plans: run_priority_schedule(tr, impl, max_plans))
    assert n >= 5
