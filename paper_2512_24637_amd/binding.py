"""ctypes binding of libmsched.so: argument marshalling only.  Every step of the
path runs in the library's HIP kernels; there is no CPU fallback, and a missing
library is an error."""
import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
NOT_RESIDENT = 0xFFFFFFFF
QUERY_STATIC_MAX = 65536
PHASES = ("expand", "count", "cut", "emit", "migrate", "plan", "host_prep", "host_launch", "host_wait", "prepare")
EXPORTED_SYMBOLS = (
    "msched_create", "msched_destroy", "msched_kernel_register", "msched_task_create",
    "msched_launch_enqueue", "msched_launch_retire", "msched_plan", "msched_migrate",
    "msched_pagetable_query", "msched_pagetable_query_static", "msched_plan_copy_lists", "msched_state_copy",
    "msched_set_profiling", "msched_get_phase_ms", "msched_strerror", "msched_last_hip_error",
    "msched_analyze", "msched_set_early_start", "msched_plan_ready_need", "msched_progress",
    "msched_gate_enqueue", "msched_gate_result",
)


class _Config(C.Structure):
    _fields_ = [("page_shift", C.c_uint32), ("n_frames", C.c_uint32), ("n_virtual_pages", C.c_uint64),
                ("hbm_pool", C.c_void_p), ("host_store", C.c_void_p), ("n_host_slots", C.c_uint64),
                ("host_slot", C.c_void_p), ("stream", C.c_void_p)]


class _Rule(C.Structure):
    _fields_ = [("kind", C.c_uint8), ("base_arg", C.c_uint8), ("n_size_args", C.c_uint8),
                ("n_stride_args", C.c_uint8), ("n_count_args", C.c_uint8),
                ("size_args", C.c_uint8 * 4), ("stride_args", C.c_uint8 * 4), ("count_args", C.c_uint8 * 4),
                ("reserved", C.c_uint8 * 7),
                ("size_coeff", C.c_uint64), ("stride_coeff", C.c_uint64), ("count_coeff", C.c_uint64)]


class _ProfileBatch(C.Structure):
    _fields_ = [("n_kernels", C.c_uint32), ("n_invocations", C.c_uint32), ("max_intervals", C.c_uint32),
                ("reserved", C.c_uint32), ("n_args", C.c_void_p), ("int64_mask", C.c_void_p),
                ("args", C.c_void_p), ("intervals", C.c_void_p), ("n_intervals", C.c_void_p)]


class _TimelineEntry(C.Structure):
    _fields_ = [("task", C.c_uint32), ("timeslice", C.c_uint32)]


class _Plan(C.Structure):
    _fields_ = [("n_evict", C.c_uint32), ("n_fetch", C.c_uint32), ("n_free_used", C.c_uint32),
                ("covered_launches", C.c_uint32), ("g_cut", C.c_uint32), ("g_end0", C.c_uint32),
                ("n_commands", C.c_uint32), ("reserved", C.c_uint32),
                ("evict_pages", C.c_void_p), ("evict_frames", C.c_void_p),
                ("fetch_pages", C.c_void_p), ("fetch_frames", C.c_void_p), ("plan_id", C.c_uint64)]


assert C.sizeof(_Rule) == 48


class MSchedError(RuntimeError):
    NAMES = {-1: "E_INVAL", -2: "E_RANGE", -3: "E_OVERFLOW", -4: "E_WSET_TOO_LARGE",
             -5: "E_STALE_PLAN", -6: "E_NOMEM", -7: "E_HIP", -8: "E_TOO_LARGE"}

    def __init__(self, code, text="", hip=0):
        self.code, self.name, self.hip = code, self.NAMES.get(code, "?"), hip
        super().__init__(f"msched error {code} ({self.name}): {text}" + (f" [hipError {hip}]" if hip else ""))


def library_path() -> str:
    return os.path.join(_PKG, "libmsched.so")


_lib = None


def load_library():
    """Load libmsched.so.  Raises if it has not been built: there is no other path."""
    global _lib
    if _lib is not None:
        return _lib
    # torch ships its own HIP runtime; it has to be the one this process loads first, or the
    # pool / stream handles torch hands over would belong to a different runtime instance
    import torch  # noqa: F401
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with paper_2512_24637_amd.build.build() "
                          "(hipcc --offload-arch=gfx950); there is no CPU fallback")
    lib = C.CDLL(path)
    vp, u32, u64 = C.c_void_p, C.c_uint32, C.c_uint64
    sig = {
        "msched_create": [C.POINTER(_Config), C.POINTER(vp)],
        "msched_destroy": [vp],
        "msched_kernel_register": [vp, C.POINTER(_Rule), u32, C.POINTER(u32)],
        "msched_task_create": [vp, C.POINTER(u32)],
        "msched_launch_enqueue": [vp, u32, u32, vp, u32, u32, vp, u32],
        "msched_launch_retire": [vp, u32, u32],
        "msched_plan": [vp, C.POINTER(_TimelineEntry), u32, C.POINTER(_Plan)],
        "msched_migrate": [vp, C.POINTER(_Plan)],
        "msched_pagetable_query": [vp, vp, u32, vp],
        "msched_pagetable_query_static": [vp, vp, u32, vp],
        "msched_plan_copy_lists": [vp, C.POINTER(_Plan), vp, vp, vp, vp],
        "msched_state_copy": [vp, vp, vp],
        "msched_set_profiling": [vp, C.c_int],
        "msched_get_phase_ms": [vp, vp],
        "msched_last_hip_error": [vp],
        "msched_analyze": [C.POINTER(_ProfileBatch), vp, vp, vp, vp],
        "msched_set_early_start": [vp, C.c_int],
        "msched_plan_ready_need": [vp, C.POINTER(_Plan), vp],
        "msched_progress": [vp, C.POINTER(u32)],
        "msched_gate_enqueue": [vp, C.POINTER(_Plan), u32, vp, u32],
        "msched_gate_result": [vp, u32, C.POINTER(u32), C.POINTER(C.c_float)],
    }
    for name, argtypes in sig.items():
        fn = getattr(lib, name)
        fn.argtypes, fn.restype = argtypes, C.c_int
    lib.msched_strerror.argtypes, lib.msched_strerror.restype = [C.c_int], C.c_char_p
    _lib = lib
    return lib


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass
class Plan:
    n_evict: int
    n_fetch: int
    n_free_used: int
    covered_launches: int
    g_cut: int
    g_end0: int
    n_commands: int
    plan_id: int
    _raw: object = None
    _owner: object = None

    def _lists(self):
        if getattr(self, "_cache", None) is None:
            self._cache = self._owner.plan_lists(self)
        return self._cache

    @property
    def evict_pages(self): return self._lists()[0]
    @property
    def evict_frames(self): return self._lists()[1]
    @property
    def fetch_pages(self): return self._lists()[2]
    @property
    def fetch_frames(self): return self._lists()[3]


class MSched:
    """One memory-scheduling context on the current GPU.

    hbm_pool / host_store are addresses of caller-owned buffers (a device tensor and a
    pinned host tensor); `stream` is a hipStream_t handle (e.g. torch's cuda_stream).
    ids_pool_ptr is the device address of the page-id pool that LIST launches index into.
    """

    def __init__(self, page_shift, n_virtual_pages, n_frames, hbm_pool_ptr, host_store_ptr,
                 n_host_slots, host_slot: Optional[np.ndarray] = None, stream: int = 0,
                 ids_pool_ptr: int = 0):
        self.lib = load_library()
        self.page_shift, self.V, self.F = int(page_shift), int(n_virtual_pages), int(n_frames)
        self._slot = None if host_slot is None else np.ascontiguousarray(host_slot, np.uint32)
        self.ids_pool_ptr = int(ids_pool_ptr)
        cfg = _Config(self.page_shift, self.F, self.V, hbm_pool_ptr, host_store_ptr, int(n_host_slots),
                      None if self._slot is None else self._slot.ctypes.data, stream or None)
        h = C.c_void_p()
        self.h = None
        self._check(self.lib.msched_create(C.byref(cfg), C.byref(h)))
        self.h = h
        self._last = None

    def _check(self, rc):
        if rc != 0:
            hip = self.lib.msched_last_hip_error(self.h)
            raise MSchedError(rc, self.lib.msched_strerror(rc).decode(), hip)

    def close(self):
        if self.h:
            self.lib.msched_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def kernel_register(self, rules: Sequence) -> int:
        arr = (_Rule * max(len(rules), 1))()
        for r, q in enumerate(rules):
            if max(len(q.size_args), len(q.stride_args), len(q.count_args)) > 4:
                raise MSchedError(-1, "more than 4 arguments in a product")
            arr[r].kind, arr[r].base_arg = q.kind, q.base_arg
            arr[r].n_size_args, arr[r].n_stride_args, arr[r].n_count_args = (
                len(q.size_args), len(q.stride_args), len(q.count_args))
            for j, a in enumerate(q.size_args): arr[r].size_args[j] = a
            for j, a in enumerate(q.stride_args): arr[r].stride_args[j] = a
            for j, a in enumerate(q.count_args): arr[r].count_args[j] = a
            arr[r].size_coeff, arr[r].stride_coeff, arr[r].count_coeff = (
                q.size_coeff, q.stride_coeff, q.count_coeff)
        kid = C.c_uint32()
        self._check(self.lib.msched_kernel_register(self.h, arr, len(rules), C.byref(kid)))
        return kid.value

    def task_create(self) -> int:
        tid = C.c_uint32()
        self._check(self.lib.msched_task_create(self.h, C.byref(tid)))
        return tid.value

    def launch_enqueue(self, task, kernel_id, args, n_args, latency=1, ids_off=0, n_ids=0, ids_ptr=None):
        a = np.zeros(12, np.uint64)
        m = min(int(n_args), 12)
        a[:m] = np.asarray(args, np.uint64)[:m]
        if ids_ptr is None:
            ids_ptr = (self.ids_pool_ptr + 4 * int(ids_off)) if n_ids else None
        self._check(self.lib.msched_launch_enqueue(self.h, task, kernel_id, _np_ptr(a), n_args, latency,
                                                   ids_ptr, n_ids))

    def launch_retire(self, task, n):
        self._check(self.lib.msched_launch_retire(self.h, task, n))

    def plan(self, timeline) -> Plan:
        n = len(timeline)
        tl = (_TimelineEntry * max(n, 1))()
        for i, (t, s) in enumerate(timeline):
            tl[i].task, tl[i].timeslice = int(t), int(s)
        raw = _Plan()
        self._check(self.lib.msched_plan(self.h, tl, n, C.byref(raw)))
        self._last = Plan(raw.n_evict, raw.n_fetch, raw.n_free_used, raw.covered_launches, raw.g_cut,
                          raw.g_end0, raw.n_commands, raw.plan_id, raw, self)
        return self._last

    def migrate(self, plan: Optional[Plan] = None):
        plan = plan or self._last
        if plan is None:
            raise MSchedError(-5, "no plan")
        plan._lists()                      # read the lists back before they can be overwritten
        self._check(self.lib.msched_migrate(self.h, C.byref(plan._raw)))

    def migrate_only(self, plan: Optional[Plan] = None):
        """migrate without first copying the lists to the host (timed runs)."""
        plan = plan or self._last
        self._check(self.lib.msched_migrate(self.h, C.byref(plan._raw)))

    def plan_lists(self, plan: Plan):
        ne, nf = plan.n_evict, plan.n_fetch
        ep, ef = np.zeros(max(ne, 1), np.uint32), np.zeros(max(ne, 1), np.uint32)
        fp, ff = np.zeros(max(nf, 1), np.uint32), np.zeros(max(nf, 1), np.uint32)
        self._check(self.lib.msched_plan_copy_lists(self.h, C.byref(plan._raw), _np_ptr(ep), _np_ptr(ef),
                                                    _np_ptr(fp), _np_ptr(ff)))
        return ep[:ne], ef[:ne], fp[:nf], ff[:nf]

    def set_early_start(self, enable: bool):
        self._check(self.lib.msched_set_early_start(self.h, int(bool(enable))))

    def ready_need(self, plan: Plan) -> np.ndarray:
        """need[g] for the covered commands of the latest plan (early start must be on)."""
        out = np.zeros(max(plan.covered_launches, 1), np.uint32)
        self._check(self.lib.msched_plan_ready_need(self.h, C.byref(plan._raw), _np_ptr(out)))
        return out[:plan.covered_launches]

    def progress(self) -> int:
        """Leading fetch entries of the latest early migration that have landed; does not wait for it."""
        v = C.c_uint32(0)
        self._check(self.lib.msched_progress(self.h, C.byref(v)))
        return int(v.value)

    def gate_enqueue(self, plan: Plan, g: int, stream: int, timeout_us: int = 0):
        """Put the device-side gate of covered command g on `stream` (a hipStream_t handle other than the context's)."""
        self._check(self.lib.msched_gate_enqueue(self.h, C.byref(plan._raw), int(g), stream, int(timeout_us)))

    def gate_result(self, g: int):
        """(status, ready_ms) of gate g: 0 not finished, 1 pages were resident, 2 gave up."""
        st, ms = C.c_uint32(0), C.c_float(0.0)
        self._check(self.lib.msched_gate_result(self.h, int(g), C.byref(st), C.byref(ms)))
        return int(st.value), float(ms.value)

    def pagetable_query(self, pages) -> np.ndarray:
        pages = np.ascontiguousarray(pages, np.uint64)
        out = np.zeros(max(pages.shape[0], 1), np.uint32)
        self._check(self.lib.msched_pagetable_query(self.h, _np_ptr(pages), pages.shape[0], _np_ptr(out)))
        return out[:pages.shape[0]]

    def pagetable_query_static(self, pages) -> np.ndarray:
        """pagetable_query through the library's static staging array (no allocation; at most QUERY_STATIC_MAX ids)."""
        pages = np.ascontiguousarray(pages, np.uint64)
        out = np.zeros(max(pages.shape[0], 1), np.uint32)
        self._check(self.lib.msched_pagetable_query_static(self.h, _np_ptr(pages), pages.shape[0], _np_ptr(out)))
        return out[:pages.shape[0]]

    def state(self):
        pt, fo = np.zeros(self.V, np.uint32), np.zeros(self.F, np.uint32)
        self._check(self.lib.msched_state_copy(self.h, _np_ptr(pt), _np_ptr(fo)))
        return pt, fo

    def set_profiling(self, level: int):
        """0 off, 1 whole-plan and migrate device times, 2 also the four planning phases."""
        self._check(self.lib.msched_set_profiling(self.h, int(level)))

    def phase_ms(self) -> dict:
        ms = np.zeros(len(PHASES), np.float32)
        self._check(self.lib.msched_get_phase_ms(self.h, _np_ptr(ms)))
        return dict(zip(PHASES, ms.tolist()))

    def slot_of(self, pages):
        pages = np.asarray(pages, np.int64)
        return pages if self._slot is None else self._slot[pages].astype(np.int64)


def rules_from_bytes(raw: np.ndarray, n_rules: np.ndarray):
    """Decode msched_analyze's rule array (uint8 [K, 8, 48]) into per-kernel lists of tuples
    (kind, base_arg, size_args, size_coeff, stride_args, stride_coeff, count_args, count_coeff)."""
    out = []
    for k in range(raw.shape[0]):
        rs = []
        for r in range(int(n_rules[k])):
            q = _Rule.from_buffer_copy(raw[k, r].tobytes())
            rs.append((q.kind, q.base_arg, tuple(q.size_args[:q.n_size_args]), q.size_coeff,
                       tuple(q.stride_args[:q.n_stride_args]), q.stride_coeff,
                       tuple(q.count_args[:q.n_count_args]), q.count_coeff))
        out.append(rs)
    return out


def analyze(n_kernels, n_invocations, max_intervals, n_args_ptr, int64_mask_ptr, args_ptr, intervals_ptr,
            n_intervals_ptr, rules_ptr, n_rules_ptr, unexplained_ptr, stream_ptr=0):
    """msched_analyze on device pointers (ints).  Asynchronous on the stream."""
    lib = load_library()
    b = _ProfileBatch(n_kernels, n_invocations, max_intervals, 0, n_args_ptr, int64_mask_ptr, args_ptr,
                      intervals_ptr, n_intervals_ptr)
    rc = lib.msched_analyze(C.byref(b), rules_ptr, n_rules_ptr, unexplained_ptr, stream_ptr or None)
    if rc != 0:
        raise MSchedError(rc, lib.msched_strerror(rc).decode(), lib.msched_last_hip_error(None))
