"""Plain-data description of a multitasking GPU workload.

A trace is what the paper's offline phase and launch interception would hand
to the memory scheduler (Sec. 4.1, Sec. 5.2): per-kernel access templates,
per-task launch records (kernel, launch arguments, profiled latency) and the
scheduler's timeslice.  It contains no page sets: deriving those is the
method's job.
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

RULE_FIXED = 1    # T1: region size is a constant
RULE_LINEAR = 2   # T2: region size = coeff * product of launch arguments
RULE_STRIDED = 3  # T3: `count` chunks of `chunk` bytes every `stride` bytes
RULE_LIST = 4     # explicit page ids attached to the launch (sparse gather)

MAX_ARGS = 12     # launch arguments per command (64-bit each)
MAX_RULES = 8     # access rules per kernel
MAX_PRODUCT_ARGS = 4


@dataclass(frozen=True)
class Rule:
    """One access rule of a kernel template.

    The region starts at launch argument ``base_arg`` (a byte address).
    ``size`` / ``stride`` / ``count`` are each ``coeff * prod(args[i] for i in idx)``
    with the empty product equal to 1.
    """
    kind: int
    base_arg: int = 0
    size_args: Tuple[int, ...] = ()
    size_coeff: int = 0
    stride_args: Tuple[int, ...] = ()
    stride_coeff: int = 0
    count_args: Tuple[int, ...] = ()
    count_coeff: int = 0


@dataclass
class TaskCommands:
    """Launch records of one task, in program order."""
    kernel_id: np.ndarray   # uint32 [n]   index into Trace.kernels
    n_args: np.ndarray      # uint32 [n]
    args: np.ndarray        # uint64 [n, MAX_ARGS]
    latency: np.ndarray     # uint32 [n]   profiled latency in ticks
    ids_off: np.ndarray     # int64  [n]   offset into Trace.ids_pool (LIST rules)
    n_ids: np.ndarray       # uint32 [n]

    def __len__(self):
        return int(self.kernel_id.shape[0])


@dataclass
class Trace:
    name: str
    page_shift: int
    n_virtual_pages: int
    n_frames: int
    timeslice: int                         # ticks per round-robin timeslice
    kernels: List[List[Rule]]
    tasks: List[TaskCommands]
    ids_pool: np.ndarray = field(default_factory=lambda: np.zeros(0, np.uint32))
    host_slot: Optional[np.ndarray] = None  # uint32 [V] page -> backing slot, or None = identity
    n_slots: int = 0                        # pages in the host backing store
    notes: str = ""
    policy: dict = field(default_factory=dict)  # parameters of a non-round-robin scheduling policy, if any
    allocations: Optional[np.ndarray] = None    # uint64 [n, 2] (start, bytes) of the buffers the tasks allocated, by start

    @property
    def page_bytes(self) -> int:
        return 1 << self.page_shift

    @property
    def n_tasks(self) -> int:
        return len(self.tasks)

    def total_launches(self) -> int:
        return sum(len(t) for t in self.tasks)


class CommandBuilder:
    """Accumulates launch records for one task."""

    def __init__(self):
        self._kid, self._nargs, self._args, self._lat, self._off, self._nids = [], [], [], [], [], []

    def add(self, kernel_id, args, latency=1, ids_off=0, n_ids=0):
        assert len(args) <= MAX_ARGS
        row = np.zeros(MAX_ARGS, np.uint64)
        row[:len(args)] = np.asarray(args, dtype=np.uint64)
        self._kid.append(kernel_id)
        self._nargs.append(len(args))
        self._args.append(row)
        self._lat.append(latency)
        self._off.append(ids_off)
        self._nids.append(n_ids)

    def build(self) -> TaskCommands:
        n = len(self._kid)
        return TaskCommands(
            kernel_id=np.asarray(self._kid, np.uint32).reshape(n),
            n_args=np.asarray(self._nargs, np.uint32).reshape(n),
            args=(np.stack(self._args) if n else np.zeros((0, MAX_ARGS), np.uint64)),
            latency=np.asarray(self._lat, np.uint32).reshape(n),
            ids_off=np.asarray(self._off, np.int64).reshape(n),
            n_ids=np.asarray(self._nids, np.uint32).reshape(n),
        )
