"""ctypes wrapper around the plain-C analyzer oracle (oracle/analyzer_oracle.c).
TEST INFRASTRUCTURE: imported by tests and the benchmark's cpu_baseline leg only."""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "analyzer_oracle.c")
_LIB = os.path.join(_HERE, "libanalyzer_oracle.so")


class _ARule(C.Structure):
    _fields_ = [("kind", C.c_int32), ("base_arg", C.c_int32), ("n_idx", C.c_int32 * 3),
                ("idx", (C.c_int32 * 4) * 3), ("coeff", C.c_uint64 * 3)]


def build(force: bool = False) -> str:
    if os.environ.get("MSCHED_ANALYZER_ORACLE_LIB"):     # a deliberately broken build, see tests/test_oracle_mutations.py
        return os.environ["MSCHED_ANALYZER_ORACLE_LIB"]
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.ana_batch.restype = None
    return _lib


def analyze(batch):
    """batch: workloads.analyzer_inputs.AnalyzerBatch.  Returns (rules, unexplained) where rules[k] is a
    list of tuples (kind, base_arg, size_args, size_coeff, stride_args, stride_coeff, count_args, count_coeff)."""
    lib = _load()
    K = batch.n_kernels
    rules = (_ARule * (K * 8))()
    n_rules = np.zeros(K, np.int32)
    unexplained = np.zeros(K, np.uint32)
    p = lambda a: a.ctypes.data_as(C.c_void_p)
    lib.ana_batch(C.c_int(K), p(batch.n_args), C.c_int(batch.n_inv), C.c_int(batch.max_iv), p(batch.ptr_mask),
                  p(batch.args), p(batch.iv), p(batch.n_iv), rules, p(n_rules), p(unexplained))
    out = []
    for k in range(K):
        rs = []
        for r in range(int(n_rules[k])):
            q = rules[k * 8 + r]
            f = [(tuple(q.idx[j][:q.n_idx[j]]), int(q.coeff[j])) for j in range(3)]
            rs.append((int(q.kind), int(q.base_arg), f[0][0], f[0][1], f[1][0], f[1][1], f[2][0], f[2][1]))
        out.append(rs)
    return out, unexplained
