"""ctypes wrapper around the plain-C oracle (oracle/msched_oracle.c).

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's
cpu_baseline leg import this.  It never imports the HIP package.
"""
import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "msched_oracle.c")
_LIB = os.path.join(_HERE, "libmsched_oracle.so")

NONE32 = 0xFFFFFFFF
ERRORS = {-1: "E_INVAL", -2: "E_RANGE", -3: "E_OVERFLOW", -4: "E_WSET_TOO_LARGE",
          -5: "E_STALE_PLAN", -6: "E_NOMEM"}


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle error {code} ({ERRORS.get(code, '?')})")
        self.code = code
        self.name = ERRORS.get(code, "?")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc if the shared object is missing or stale.  MSCHED_ORACLE_LIB names a
    library to load instead (tests/test_oracle_mutations.py points it at deliberately broken builds to
    show that the pins notice)."""
    if os.environ.get("MSCHED_ORACLE_LIB"):
        return os.environ["MSCHED_ORACLE_LIB"]
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", _LIB, _SRC])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = C.CDLL(build())
    u32p, u64p, i32p, u8p = (C.POINTER(C.c_uint32), C.POINTER(C.c_uint64), C.POINTER(C.c_int),
                             C.POINTER(C.c_uint8))
    lib.orc_create.restype = C.c_void_p
    lib.orc_create.argtypes = [C.c_int, C.c_uint64, C.c_uint32, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]
    lib.orc_destroy.argtypes = [C.c_void_p]
    lib.orc_destroy.restype = None
    lib.orc_kernel_register.argtypes = [C.c_void_p, C.c_int, i32p, i32p, i32p, i32p, u64p]
    lib.orc_task_create.argtypes = [C.c_void_p]
    lib.orc_launch_enqueue.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_uint32,
                                       C.c_uint32, C.c_void_p, C.c_uint32]
    lib.orc_launch_retire.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32]
    lib.orc_command_pages.restype = C.c_int64
    lib.orc_command_pages.argtypes = [C.c_void_p, C.c_uint32, C.c_uint64, C.c_void_p, C.c_uint64]
    lib.orc_plan.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32]
    lib.orc_plan_counts.argtypes = [C.c_void_p, C.c_void_p]
    lib.orc_plan_lists.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.orc_migrate.argtypes = [C.c_void_p]
    lib.orc_ready_need.argtypes = [C.c_void_p, C.c_void_p]
    lib.orc_migrate_prefix.argtypes = [C.c_void_p, C.c_uint32]
    lib.orc_demand_touch.restype = C.c_int64
    lib.orc_demand_touch.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32]
    lib.orc_pagetable_query.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p]
    lib.orc_state.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    lib.orc_state.restype = None
    lib.orc_lru_faults.restype = C.c_int64
    lib.orc_lru_faults.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32]
    _lib = lib
    return lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass
class OraclePlan:
    n_fetch: int
    n_evict: int
    n_free_used: int
    g_cut: int
    g_end0: int
    n_commands: int
    covered_launches: int
    evict_pages: np.ndarray
    evict_frames: np.ndarray
    fetch_pages: np.ndarray
    fetch_frames: np.ndarray


class Oracle:
    """One memory-scheduling context on the CPU.

    with_bytes=True keeps byte images of the HBM pool and the host backing
    store (numpy uint64 views in `.pool_words` / `.host_words`, one row per
    frame / slot); otherwise only metadata is tracked.
    """

    def __init__(self, page_shift, n_virtual_pages, n_frames, host_slot=None, n_slots=0,
                 with_bytes=False, ids_pool=None):
        self.lib = _load()
        self.page_shift, self.V, self.F = int(page_shift), int(n_virtual_pages), int(n_frames)
        self._slot = None if host_slot is None else np.ascontiguousarray(host_slot, np.uint32)
        self.n_slots = int(n_slots) if host_slot is not None else self.V
        self.ids_pool = None if ids_pool is None else np.ascontiguousarray(ids_pool, np.uint32)
        self.pool_words = self.host_words = None
        if with_bytes:
            wpp = (1 << self.page_shift) // 8
            self.pool_words = np.zeros((self.F, wpp), np.uint64)
            self.host_words = np.zeros((self.n_slots, wpp), np.uint64)
        self.h = self.lib.orc_create(self.page_shift, self.V, self.F, _ptr(self._slot), self.n_slots,
                                     _ptr(self.pool_words), _ptr(self.host_words))
        if not self.h:
            raise OracleError(-1)

    @classmethod
    def for_trace(cls, trace, with_bytes=False):
        return cls(trace.page_shift, trace.n_virtual_pages, trace.n_frames, trace.host_slot,
                   trace.n_slots, with_bytes, trace.ids_pool)

    def close(self):
        if self.h:
            self.lib.orc_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @staticmethod
    def _check(rc):
        if rc < 0:
            raise OracleError(int(rc))
        return int(rc)

    def kernel_register(self, rules) -> int:
        n = len(rules)
        kind = np.zeros(max(n, 1), np.int32)
        base = np.zeros(max(n, 1), np.int32)
        n_idx = np.zeros((max(n, 1), 3), np.int32)
        idx = np.zeros((max(n, 1), 3, 4), np.int32)
        coeff = np.zeros((max(n, 1), 3), np.uint64)
        for r, q in enumerate(rules):
            kind[r], base[r] = q.kind, q.base_arg
            for f, (ix, co) in enumerate(((q.size_args, q.size_coeff), (q.stride_args, q.stride_coeff),
                                          (q.count_args, q.count_coeff))):
                if len(ix) > 4:
                    raise OracleError(-1)
                n_idx[r, f] = len(ix)
                idx[r, f, :len(ix)] = ix
                coeff[r, f] = co
        ip = lambda a: a.ctypes.data_as(C.POINTER(C.c_int))
        return self._check(self.lib.orc_kernel_register(
            self.h, n, ip(kind), ip(base), ip(n_idx), ip(idx), coeff.ctypes.data_as(C.POINTER(C.c_uint64))))

    def task_create(self) -> int:
        return self._check(self.lib.orc_task_create(self.h))

    def launch_enqueue(self, task, kernel_id, args, n_args, latency=1, ids_off=0, n_ids=0, ids=None):
        a = np.zeros(12, np.uint64)
        a[:min(n_args, 12)] = np.asarray(args, np.uint64)[:min(n_args, 12)]
        if ids is None and n_ids:
            ids = self.ids_pool[ids_off:ids_off + n_ids]
        if ids is not None:
            ids = np.ascontiguousarray(ids, np.uint32)
            n_ids = ids.shape[0]
        self._check(self.lib.orc_launch_enqueue(self.h, task, kernel_id, _ptr(a), n_args, latency,
                                                _ptr(ids), n_ids))

    def launch_retire(self, task, n):
        self._check(self.lib.orc_launch_retire(self.h, task, n))

    def command_pages(self, task, index) -> np.ndarray:
        n = self._check(self.lib.orc_command_pages(self.h, task, index, None, 0))
        out = np.zeros(max(n, 1), np.uint32)
        self._check(self.lib.orc_command_pages(self.h, task, index, _ptr(out), n))
        return out[:n]

    def plan(self, timeline) -> OraclePlan:
        tl = np.asarray(timeline, np.uint32).reshape(-1, 2)
        tasks = np.ascontiguousarray(tl[:, 0])
        slices = np.ascontiguousarray(tl[:, 1])
        self._check(self.lib.orc_plan(self.h, _ptr(tasks), _ptr(slices), tl.shape[0]))
        c = np.zeros(8, np.uint32)
        self._check(self.lib.orc_plan_counts(self.h, _ptr(c)))
        nf, ne = int(c[0]), int(c[1])
        ep, ef = np.zeros(max(ne, 1), np.uint32), np.zeros(max(ne, 1), np.uint32)
        fp, ff = np.zeros(max(nf, 1), np.uint32), np.zeros(max(nf, 1), np.uint32)
        self._check(self.lib.orc_plan_lists(self.h, _ptr(ep), _ptr(ef), _ptr(fp), _ptr(ff)))
        return OraclePlan(nf, ne, int(c[2]), int(c[3]), int(c[4]), int(c[5]), int(c[6]),
                          ep[:ne], ef[:ne], fp[:nf], ff[:nf])

    def migrate(self):
        self._check(self.lib.orc_migrate(self.h))

    def ready_need(self, g_cut) -> np.ndarray:
        """need[g]: leading fetch entries that must have landed before covered command g may start."""
        out = np.zeros(max(int(g_cut), 1), np.uint32)
        self._check(self.lib.orc_ready_need(self.h, _ptr(out)))
        return out[:int(g_cut)]

    def migrate_prefix(self, n):
        """Carry out the pending plan up to fetch entry n - 1 (in list order)."""
        self._check(self.lib.orc_migrate_prefix(self.h, int(n)))

    def demand_touch(self, pages) -> int:
        """The running command touches these pages; the ones that are not resident fault in.  Returns the faults."""
        pages = np.ascontiguousarray(pages, np.uint32)
        return self._check(self.lib.orc_demand_touch(self.h, _ptr(pages), pages.shape[0]))

    def pagetable_query(self, pages) -> np.ndarray:
        pages = np.ascontiguousarray(pages, np.uint64)
        out = np.zeros(max(pages.shape[0], 1), np.uint32)
        self._check(self.lib.orc_pagetable_query(self.h, _ptr(pages), pages.shape[0], _ptr(out)))
        return out[:pages.shape[0]]

    def state(self):
        pt, fo = np.zeros(self.V, np.uint32), np.zeros(self.F, np.uint32)
        self.lib.orc_state(self.h, _ptr(pt), _ptr(fo))
        return pt, fo

    def lru_faults(self, tasks, indices, capacity) -> int:
        t = np.ascontiguousarray(tasks, np.uint32)
        i = np.ascontiguousarray(indices, np.uint64)
        return self._check(self.lib.orc_lru_faults(self.h, _ptr(t), _ptr(i), t.shape[0], capacity))

    def slot_of(self, pages):
        pages = np.asarray(pages, np.int64)
        return pages if self._slot is None else self._slot[pages].astype(np.int64)
