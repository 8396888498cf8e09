"""ctypes binding of the C-ABI library (`include/fikit.h`).

Argument marshalling only: tensors in, tensors out; every step of the path runs in the library's
HIP kernels.  PyTorch provides device memory and the stream.  There is no fallback: if the
library is missing or cannot be loaded, importing the functions fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import NamedTuple, Optional

import numpy as np
import torch

from . import build as _build

FIKIT_OK = 0
FIKIT_INVALID_ARG = -1
FIKIT_WORKSPACE_TOO_SMALL = -2
FIKIT_ROW_CAPACITY = -3
FIKIT_BAD_RECORD = -4
FIKIT_UNKNOWN_ID = -5
FIKIT_HIP_ERROR = -6
FIKIT_UNSUPPORTED = -7
FIKIT_TOO_LARGE = -8
FIKIT_STATIC_MAX_IDS = 1 << 20
FIKIT_STATIC_MAX_TASKS = 16384
FIKIT_PREDICT_P50, FIKIT_PREDICT_MEAN = 0, 1

EXPORTS = ("fikit_profile_workspace_bytes", "fikit_profile", "fikit_gapfill_workspace_bytes",
           "fikit_gapfill", "fikit_profile_gapfill_workspace_bytes", "fikit_profile_gapfill", "fikit_gapfill_static", "fikit_measure_workspace_bytes", "fikit_measure", "fikit_replay_workspace_bytes",
           "fikit_gapfill_replay", "fikit_prio_fill_workspace_bytes", "fikit_prio_fill", "fikit_pairing_workspace_bytes",
           "fikit_pairing_best", "fikit_profile_merge_workspace_bytes", "fikit_profile_merge", "fikit_status_string", "fikit_version", "fikit_set_wait_limit",
           "fikit_trace_enable", "fikit_trace_read")

# Layout of a profile row as seen from numpy (128 bytes; see fikit_row in fikit.h).
STATS_DTYPE = np.dtype([("count", "<u8"), ("sum", "<u8"), ("min", "<i8"), ("max", "<i8"),
                        ("p50", "<i8"), ("p95", "<i8")])
ROW_DTYPE = np.dtype([("kernel_id", "<u8"), ("task", "<u4"), ("reserved0", "<u4"),
                      ("exec", STATS_DTYPE), ("gap", STATS_DTYPE), ("reserved1", "u1", (16,))])
ROW_BYTES = 128
LAUNCH_BYTES = 64


class FikitError(RuntimeError):
    def __init__(self, status: int, what: str, n_rows: Optional[int] = None):
        super().__init__(f"{what}: status {status} ({status_string(status)})")
        self.status = status
        self.n_rows = n_rows


class _GapfillParams(ctypes.Structure):
    _fields_ = [("margin_ns", ctypes.c_int64), ("min_gap_ns", ctypes.c_int64), ("predictor", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class _ReplayParams(ctypes.Structure):
    _fields_ = [("margin_ns", ctypes.c_int64), ("min_gap_ns", ctypes.c_int64), ("feedback", ctypes.c_int32),
                ("predictor", ctypes.c_int32)]


_lib = None


def library_path() -> str:
    return _build.LIB


def load() -> ctypes.CDLL:
    """Loads the built library (building it first only if no library file exists)."""
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            _build.build_library()
        lib = ctypes.CDLL(path)
        vp, u64, u32, sz = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_size_t
        lib.fikit_profile_workspace_bytes.restype = sz
        lib.fikit_profile_workspace_bytes.argtypes = [u64, u32]
        lib.fikit_profile.restype = ctypes.c_int
        lib.fikit_profile.argtypes = [vp, u64, vp, u32, vp, vp, u64, vp, ctypes.POINTER(u64), vp, sz, vp]
        lib.fikit_gapfill_workspace_bytes.restype = sz
        lib.fikit_gapfill_workspace_bytes.argtypes = [u64, u32, u64]
        lib.fikit_gapfill.restype = ctypes.c_int
        lib.fikit_gapfill.argtypes = [vp, vp, u32, vp, vp, vp, vp, u64, ctypes.POINTER(_GapfillParams), vp,
                                      vp, vp, vp, vp, vp, sz, vp]
        lib.fikit_profile_gapfill_workspace_bytes.restype = sz
        lib.fikit_profile_gapfill_workspace_bytes.argtypes = [u64, u32, u64]
        lib.fikit_profile_gapfill.restype = ctypes.c_int
        lib.fikit_profile_gapfill.argtypes = [vp, u64, vp, u32, vp, vp, u64, vp, ctypes.POINTER(u64), vp, vp, u64,
                                              ctypes.POINTER(_GapfillParams), vp, vp, vp, vp, vp, vp, sz, vp]
        lib.fikit_gapfill_static.restype = ctypes.c_int
        lib.fikit_gapfill_static.argtypes = [vp, u64, vp, u32, vp, vp, vp, vp, u64, ctypes.POINTER(_GapfillParams), vp, u64,
                                             vp, vp, vp, vp, vp, vp]
        lib.fikit_measure_workspace_bytes.restype = sz
        lib.fikit_measure_workspace_bytes.argtypes = []
        lib.fikit_measure.restype = ctypes.c_int
        lib.fikit_measure.argtypes = [vp, u64, vp, u32, vp, vp, vp, sz, vp]
        lib.fikit_replay_workspace_bytes.restype = sz
        lib.fikit_replay_workspace_bytes.argtypes = [u64, u32, u64]
        lib.fikit_prio_fill_workspace_bytes.restype = sz
        lib.fikit_prio_fill_workspace_bytes.argtypes = [u64, u32, u64]
        lib.fikit_prio_fill.restype = ctypes.c_int
        lib.fikit_prio_fill.argtypes = [vp, vp, u32, vp, vp, vp, vp, vp, vp, u64, ctypes.POINTER(_GapfillParams), vp,
                                        vp, vp, vp, vp, vp, sz, vp]
        lib.fikit_pairing_workspace_bytes.restype = sz
        lib.fikit_pairing_workspace_bytes.argtypes = [u32]
        lib.fikit_pairing_best.restype = ctypes.c_int
        lib.fikit_pairing_best.argtypes = [vp, vp, u64, u32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.fikit_profile_merge_workspace_bytes.restype = sz
        lib.fikit_profile_merge_workspace_bytes.argtypes = [u32]
        lib.fikit_profile_merge.restype = ctypes.c_int
        lib.fikit_profile_merge.argtypes = [vp, vp, vp, vp, u32, vp, u64, vp, ctypes.POINTER(ctypes.c_uint64), vp, sz, vp]
        lib.fikit_gapfill_replay.restype = ctypes.c_int
        lib.fikit_gapfill_replay.argtypes = [vp, vp, u32, vp, vp, vp, vp, vp, u64, ctypes.POINTER(_ReplayParams), vp,
                                             vp, vp, vp, vp, vp, sz, vp]
        lib.fikit_status_string.restype = ctypes.c_char_p
        lib.fikit_status_string.argtypes = [ctypes.c_int]
        lib.fikit_version.restype = ctypes.c_int
        lib.fikit_version.argtypes = []
        lib.fikit_set_wait_limit.restype = None
        lib.fikit_set_wait_limit.argtypes = [ctypes.c_uint32]
        lib.fikit_trace_enable.restype = None
        lib.fikit_trace_enable.argtypes = [ctypes.c_int]
        lib.fikit_trace_read.restype = ctypes.c_int
        lib.fikit_trace_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_char_p),
                                         ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)]
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().fikit_status_string(status).decode()


def fikit_set_wait_limit(polls: int) -> None:
    load().fikit_set_wait_limit(polls)


def fikit_trace_enable(on: bool) -> None:
    load().fikit_trace_enable(1 if on else 0)


def fikit_trace_read() -> dict:
    """{name: (total_ms, intervals)} accumulated since fikit_trace_enable(True)."""
    lib = load()
    out = {}
    n = lib.fikit_trace_read(-1, None, None, None)
    for i in range(n):
        name, ms, k = ctypes.c_char_p(), ctypes.c_double(), ctypes.c_int()
        lib.fikit_trace_read(i, ctypes.byref(name), ctypes.byref(ms), ctypes.byref(k))
        out[name.value.decode()] = (ms.value, k.value)
    return out


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_handle(stream: Optional[torch.cuda.Stream]):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def fikit_profile_workspace_bytes(n_records: int, n_tasks: int) -> int:
    return int(load().fikit_profile_workspace_bytes(n_records, n_tasks))


def fikit_gapfill_workspace_bytes(n_ids: int, n_tasks: int, n_scenarios: int) -> int:
    return int(load().fikit_gapfill_workspace_bytes(n_ids, n_tasks, n_scenarios))


def workspace(nbytes: int, device) -> torch.Tensor:
    """A device buffer of at least nbytes (torch allocations are 256-byte aligned or better)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


class Profile(NamedTuple):
    ids: torch.Tensor               # int64 view of the uint64 Kernel IDs, launch order
    rows: torch.Tensor              # uint8 [n_rows, 128]
    task_row_offsets: torch.Tensor  # int64 [n_tasks + 1]
    n_rows: int


def fikit_profile(records: torch.Tensor, task_offsets: torch.Tensor, *, row_capacity: Optional[int] = None,
                  ids_out: Optional[torch.Tensor] = None, rows_out: Optional[torch.Tensor] = None,
                  task_row_offsets_out: Optional[torch.Tensor] = None, workspace_buf: Optional[torch.Tensor] = None,
                  want_ids: bool = True, stream: Optional[torch.cuda.Stream] = None) -> Profile:
    """records: uint8 [n, 64] device tensor of launch records; task_offsets: int64 [T+1] device
    tensor holding the uint64 CSR offsets.  Output tensors are allocated unless given."""
    lib = load()
    dev = records.device
    assert records.dtype == torch.uint8 and records.is_contiguous()
    n = records.numel() // LAUNCH_BYTES
    assert records.numel() == n * LAUNCH_BYTES
    assert task_offsets.dtype == torch.int64 and task_offsets.is_contiguous() and task_offsets.device == dev
    n_tasks = task_offsets.numel() - 1
    if row_capacity is None:
        row_capacity = rows_out.shape[0] if rows_out is not None else n
    if ids_out is None and want_ids:
        ids_out = torch.empty(n, dtype=torch.int64, device=dev)
    if rows_out is None:
        rows_out = torch.empty((row_capacity, ROW_BYTES), dtype=torch.uint8, device=dev)
    if task_row_offsets_out is None:
        task_row_offsets_out = torch.empty(n_tasks + 1, dtype=torch.int64, device=dev)
    need = fikit_profile_workspace_bytes(n, n_tasks)
    if workspace_buf is None:
        workspace_buf = workspace(need, dev)
    n_rows = ctypes.c_uint64(0)
    with torch.cuda.device(dev):
        st = lib.fikit_profile(_ptr(records), n, _ptr(task_offsets), n_tasks, _ptr(ids_out), _ptr(rows_out),
                               row_capacity, _ptr(task_row_offsets_out), ctypes.byref(n_rows),
                               _ptr(workspace_buf), workspace_buf.numel(), _stream_handle(stream))
    if st != FIKIT_OK:
        raise FikitError(st, "fikit_profile", int(n_rows.value))
    return Profile(ids_out, rows_out[: int(n_rows.value)], task_row_offsets_out, int(n_rows.value))


class GapFill(NamedTuple):
    fill_count: torch.Tensor        # int32 view of uint32 [n_gaps]
    filled_ns: torch.Tensor         # int64 [n_gaps]
    lp_completion_ns: torch.Tensor  # int64 [S]
    lp_placed: torch.Tensor         # int64 view of uint64 [S]


def fikit_gapfill(ids: torch.Tensor, task_offsets: torch.Tensor, rows: torch.Tensor, task_row_offsets: torch.Tensor,
                  hp_task: torch.Tensor, lp_task: torch.Tensor, gap_offsets: torch.Tensor, *, margin_ns: int,
                  min_gap_ns: int, predictor: int = FIKIT_PREDICT_P50, n_gaps: Optional[int] = None,
                  n_ids: Optional[int] = None, out: Optional[GapFill] = None, workspace_buf: Optional[torch.Tensor] = None,
                  stream: Optional[torch.cuda.Stream] = None) -> GapFill:
    """hp_task / lp_task: int32 views of the uint32 task numbers; gap_offsets: int64 [S+1]."""
    lib = load()
    dev = task_offsets.device
    n_tasks = task_offsets.numel() - 1
    s = hp_task.numel()
    assert hp_task.dtype == torch.int32 and lp_task.dtype == torch.int32 and lp_task.numel() == s
    assert gap_offsets.dtype == torch.int64 and gap_offsets.numel() == s + 1
    for t in (ids, task_offsets, rows, task_row_offsets, hp_task, lp_task, gap_offsets):
        assert t.is_contiguous() and t.device == dev
    if n_gaps is None:
        n_gaps = int(gap_offsets[-1].item()) if s else 0
    if n_ids is None:
        n_ids = ids.numel()
    if out is None:
        out = GapFill(torch.empty(n_gaps, dtype=torch.int32, device=dev),
                      torch.empty(n_gaps, dtype=torch.int64, device=dev),
                      torch.empty(s, dtype=torch.int64, device=dev),
                      torch.empty(s, dtype=torch.int64, device=dev))
    need = fikit_gapfill_workspace_bytes(n_ids, n_tasks, s)
    if workspace_buf is None:
        workspace_buf = workspace(need, dev)
    params = _GapfillParams(margin_ns, min_gap_ns, predictor, 0)
    with torch.cuda.device(dev):
        st = lib.fikit_gapfill(_ptr(ids), _ptr(task_offsets), n_tasks, _ptr(rows), _ptr(task_row_offsets),
                               _ptr(hp_task), _ptr(lp_task), s, ctypes.byref(params), _ptr(gap_offsets),
                               _ptr(out.fill_count), _ptr(out.filled_ns), _ptr(out.lp_completion_ns),
                               _ptr(out.lp_placed), _ptr(workspace_buf), workspace_buf.numel(),
                               _stream_handle(stream))
    if st != FIKIT_OK:
        raise FikitError(st, "fikit_gapfill")
    return out


def fikit_profile_gapfill_workspace_bytes(n_records: int, n_tasks: int, n_scenarios: int) -> int:
    return int(load().fikit_profile_gapfill_workspace_bytes(n_records, n_tasks, n_scenarios))


def fikit_profile_gapfill(records: torch.Tensor, task_offsets: torch.Tensor, hp_task: torch.Tensor, lp_task: torch.Tensor,
                          gap_offsets: torch.Tensor, *, margin_ns: int, min_gap_ns: int, predictor: int = FIKIT_PREDICT_P50,
                          n_gaps: Optional[int] = None, row_capacity: Optional[int] = None,
                          ids_out: Optional[torch.Tensor] = None, rows_out: Optional[torch.Tensor] = None,
                          task_row_offsets_out: Optional[torch.Tensor] = None, out: Optional[GapFill] = None,
                          workspace_buf: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """fikit_profile and fikit_gapfill as one call -> (Profile, GapFill).  Arguments as in the two."""
    lib = load()
    dev = records.device
    assert records.dtype == torch.uint8 and records.is_contiguous()
    n = records.numel() // LAUNCH_BYTES
    assert records.numel() == n * LAUNCH_BYTES
    n_tasks = task_offsets.numel() - 1
    s = hp_task.numel()
    assert hp_task.dtype == torch.int32 and lp_task.dtype == torch.int32 and lp_task.numel() == s
    assert gap_offsets.dtype == torch.int64 and gap_offsets.numel() == s + 1
    for t in (task_offsets, hp_task, lp_task, gap_offsets):
        assert t.is_contiguous() and t.device == dev
    if n_gaps is None:
        n_gaps = int(gap_offsets[-1].item()) if s else 0
    if row_capacity is None:
        row_capacity = rows_out.shape[0] if rows_out is not None else n
    if ids_out is None:
        ids_out = torch.empty(n, dtype=torch.int64, device=dev)
    if rows_out is None:
        rows_out = torch.empty((row_capacity, ROW_BYTES), dtype=torch.uint8, device=dev)
    if task_row_offsets_out is None:
        task_row_offsets_out = torch.empty(n_tasks + 1, dtype=torch.int64, device=dev)
    if out is None:
        out = GapFill(torch.empty(n_gaps, dtype=torch.int32, device=dev),
                      torch.empty(n_gaps, dtype=torch.int64, device=dev),
                      torch.empty(s, dtype=torch.int64, device=dev),
                      torch.empty(s, dtype=torch.int64, device=dev))
    if workspace_buf is None:
        workspace_buf = workspace(fikit_profile_gapfill_workspace_bytes(n, n_tasks, s), dev)
    params = _GapfillParams(margin_ns, min_gap_ns, predictor, 0)
    n_rows = ctypes.c_uint64(0)
    with torch.cuda.device(dev):
        st = lib.fikit_profile_gapfill(_ptr(records), n, _ptr(task_offsets), n_tasks, _ptr(ids_out), _ptr(rows_out), row_capacity,
                                       _ptr(task_row_offsets_out), ctypes.byref(n_rows), _ptr(hp_task), _ptr(lp_task), s,
                                       ctypes.byref(params), _ptr(gap_offsets), _ptr(out.fill_count), _ptr(out.filled_ns),
                                       _ptr(out.lp_completion_ns), _ptr(out.lp_placed), _ptr(workspace_buf),
                                       workspace_buf.numel(), _stream_handle(stream))
    if st != FIKIT_OK:
        raise FikitError(st, "fikit_profile_gapfill", int(n_rows.value))
    return Profile(ids_out, rows_out[: int(n_rows.value)], task_row_offsets_out, int(n_rows.value)), out


def fikit_gapfill_static(ids: torch.Tensor, task_offsets: torch.Tensor, rows: torch.Tensor, task_row_offsets: torch.Tensor,
                         hp_task: torch.Tensor, lp_task: torch.Tensor, gap_offsets: torch.Tensor, *, n_ids: int, n_gaps: int,
                         margin_ns: int, min_gap_ns: int, out: GapFill, status_out: torch.Tensor,
                         predictor: int = FIKIT_PREDICT_P50, stream: Optional[torch.cuda.Stream] = None) -> None:
    """fikit_gapfill on the library's built-in scratch buffer.  Every buffer, including the outputs and the int32
    status word, is the caller's; nothing is allocated, nothing is waited for: read status_out after synchronising."""
    lib = load()
    dev = task_offsets.device
    n_tasks = task_offsets.numel() - 1
    s = hp_task.numel()
    assert status_out.dtype == torch.int32 and status_out.numel() >= 1 and status_out.device == dev
    params = _GapfillParams(margin_ns, min_gap_ns, predictor, 0)
    with torch.cuda.device(dev):
        st = lib.fikit_gapfill_static(_ptr(ids), n_ids, _ptr(task_offsets), n_tasks, _ptr(rows), _ptr(task_row_offsets),
                                      _ptr(hp_task), _ptr(lp_task), s, ctypes.byref(params), _ptr(gap_offsets), n_gaps,
                                      _ptr(out.fill_count), _ptr(out.filled_ns), _ptr(out.lp_completion_ns),
                                      _ptr(out.lp_placed), _ptr(status_out), _stream_handle(stream))
    if st != FIKIT_OK:
        raise FikitError(st, "fikit_gapfill_static")


def fikit_measure_workspace_bytes() -> int:
    return int(load().fikit_measure_workspace_bytes())


def fikit_measure(records: torch.Tensor, task_offsets: torch.Tensor, *, exec_out: Optional[torch.Tensor] = None,
                  gap_out: Optional[torch.Tensor] = None, workspace_buf: Optional[torch.Tensor] = None,
                  stream: Optional[torch.cuda.Stream] = None):
    """-> (exec_ns, gap_ns): int64 [n] device tensors (gap_ns is -1 for the last launch of a task)."""
    lib = load()
    dev = records.device
    assert records.dtype == torch.uint8 and records.is_contiguous()
    n = records.numel() // LAUNCH_BYTES
    assert task_offsets.dtype == torch.int64 and task_offsets.is_contiguous() and task_offsets.device == dev
    n_tasks = task_offsets.numel() - 1
    if exec_out is None:
        exec_out = torch.empty(n, dtype=torch.int64, device=dev)
    if gap_out is None:
        gap_out = torch.empty(n, dtype=torch.int64, device=dev)
    if workspace_buf is None:
        workspace_buf = workspace(fikit_measure_workspace_bytes(), dev)
    with torch.cuda.device(dev):
        st = lib.fikit_measure(_ptr(records), n, _ptr(task_offsets), n_tasks, _ptr(exec_out), _ptr(gap_out),
                               _ptr(workspace_buf), workspace_buf.numel(), _stream_handle(stream))
    if st != FIKIT_OK:
        raise FikitError(st, "fikit_measure")
    return exec_out, gap_out


class Replay(NamedTuple):
    fill_count: torch.Tensor   # int32 view of uint32 [n_gaps]
    filled_ns: torch.Tensor    # int64 [n_gaps]
    hp_delay_ns: torch.Tensor  # int64 [S]
    lp_placed: torch.Tensor    # int64 view of uint64 [S]


def fikit_replay_workspace_bytes(n_ids: int, n_tasks: int, n_scenarios: int) -> int:
    return int(load().fikit_replay_workspace_bytes(n_ids, n_tasks, n_scenarios))


def fikit_gapfill_replay(ids: torch.Tensor, task_offsets: torch.Tensor, rows: torch.Tensor, task_row_offsets: torch.Tensor,
                         actual_gap_ns: torch.Tensor, hp_task: torch.Tensor, lp_task: torch.Tensor,
                         gap_offsets: torch.Tensor, *, margin_ns: int, min_gap_ns: int, feedback: bool,
                         predictor: int = FIKIT_PREDICT_P50, n_gaps: Optional[int] = None, n_ids: Optional[int] = None, out: Optional[Replay] = None,
                         workspace_buf: Optional[torch.Tensor] = None,
                         stream: Optional[torch.cuda.Stream] = None) -> Replay:
    """As fikit_gapfill, plus actual_gap_ns: int64 [n_ids] (fikit_measure's gap_ns)."""
    lib = load()
    dev = task_offsets.device
    n_tasks = task_offsets.numel() - 1
    s = hp_task.numel()
    assert hp_task.dtype == torch.int32 and lp_task.dtype == torch.int32 and lp_task.numel() == s
    assert gap_offsets.dtype == torch.int64 and gap_offsets.numel() == s + 1
    assert actual_gap_ns.dtype == torch.int64
    for t in (ids, task_offsets, rows, task_row_offsets, actual_gap_ns, hp_task, lp_task, gap_offsets):
        assert t.is_contiguous() and t.device == dev
    if n_gaps is None:
        n_gaps = int(gap_offsets[-1].item()) if s else 0
    if n_ids is None:
        n_ids = ids.numel()
    if out is None:
        out = Replay(torch.empty(n_gaps, dtype=torch.int32, device=dev), torch.empty(n_gaps, dtype=torch.int64, device=dev),
                     torch.empty(s, dtype=torch.int64, device=dev), torch.empty(s, dtype=torch.int64, device=dev))
    if workspace_buf is None:
        workspace_buf = workspace(fikit_replay_workspace_bytes(n_ids, n_tasks, s), dev)
    params = _ReplayParams(margin_ns, min_gap_ns, 1 if feedback else 0, predictor)
    with torch.cuda.device(dev):
        st = lib.fikit_gapfill_replay(_ptr(ids), _ptr(task_offsets), n_tasks, _ptr(rows), _ptr(task_row_offsets),
                                      _ptr(actual_gap_ns), _ptr(hp_task), _ptr(lp_task), s, ctypes.byref(params),
                                      _ptr(gap_offsets), _ptr(out.fill_count), _ptr(out.filled_ns), _ptr(out.hp_delay_ns),
                                      _ptr(out.lp_placed), _ptr(workspace_buf), workspace_buf.numel(),
                                      _stream_handle(stream))
    if st != FIKIT_OK:
        raise FikitError(st, "fikit_gapfill_replay")
    return out


class PrioFill(NamedTuple):
    fill_count: torch.Tensor     # int32 view of uint32 [n_gaps]
    filled_ns: torch.Tensor      # int64 [n_gaps]
    lp_placed: torch.Tensor      # int64 view of uint64 [n_entries]
    lp_placed_ns: torch.Tensor   # int64 [n_entries]


FIKIT_PRIO_MAX_LP = 64


def fikit_prio_fill_workspace_bytes(n_ids: int, n_tasks: int, n_scenarios: int) -> int:
    return int(load().fikit_prio_fill_workspace_bytes(n_ids, n_tasks, n_scenarios))


def fikit_prio_fill(ids: torch.Tensor, task_offsets: torch.Tensor, rows: torch.Tensor, task_row_offsets: torch.Tensor,
                    hp_task: torch.Tensor, lp_offsets: torch.Tensor, lp_task: torch.Tensor, lp_prio: torch.Tensor,
                    gap_offsets: torch.Tensor, *, margin_ns: int, min_gap_ns: int, predictor: int = FIKIT_PREDICT_P50,
                    n_gaps: Optional[int] = None, n_ids: Optional[int] = None, out: Optional[PrioFill] = None,
                    workspace_buf: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> PrioFill:
    """hp_task: int32 [S]; lp_offsets: int64 [S+1]; lp_task, lp_prio: int32 [n_entries]; gap_offsets: int64 [S+1]."""
    lib = load()
    dev = task_offsets.device
    n_tasks = task_offsets.numel() - 1
    s = hp_task.numel()
    n_entries = lp_task.numel()
    assert hp_task.dtype == torch.int32 and lp_task.dtype == torch.int32 and lp_prio.dtype == torch.int32
    assert lp_prio.numel() == n_entries
    assert lp_offsets.dtype == torch.int64 and lp_offsets.numel() == s + 1
    assert gap_offsets.dtype == torch.int64 and gap_offsets.numel() == s + 1
    for t in (ids, task_offsets, rows, task_row_offsets, hp_task, lp_offsets, lp_task, lp_prio, gap_offsets):
        assert t.is_contiguous() and t.device == dev
    if n_gaps is None:
        n_gaps = int(gap_offsets[-1].item()) if s else 0
    if n_ids is None:
        n_ids = ids.numel()
    if out is None:
        out = PrioFill(torch.empty(n_gaps, dtype=torch.int32, device=dev), torch.empty(n_gaps, dtype=torch.int64, device=dev),
                       torch.empty(n_entries, dtype=torch.int64, device=dev),
                       torch.empty(n_entries, dtype=torch.int64, device=dev))
    if workspace_buf is None:
        workspace_buf = workspace(fikit_prio_fill_workspace_bytes(n_ids, n_tasks, s), dev)
    params = _GapfillParams(margin_ns, min_gap_ns, predictor, 0)
    with torch.cuda.device(dev):
        st = lib.fikit_prio_fill(_ptr(ids), _ptr(task_offsets), n_tasks, _ptr(rows), _ptr(task_row_offsets), _ptr(hp_task),
                                 _ptr(lp_offsets), _ptr(lp_task), _ptr(lp_prio), s, ctypes.byref(params), _ptr(gap_offsets),
                                 _ptr(out.fill_count), _ptr(out.filled_ns), _ptr(out.lp_placed), _ptr(out.lp_placed_ns),
                                 _ptr(workspace_buf), workspace_buf.numel(), _stream_handle(stream))
    if st != FIKIT_OK:
        raise FikitError(st, "fikit_prio_fill")
    return out


class Pairing(NamedTuple):
    scenario_filled_ns: torch.Tensor  # int64 [S]
    best_scenario: torch.Tensor       # int64 view of uint64 [n_tasks] (-1 = the task heads no scenario)
    best_lp: torch.Tensor             # int32 view of uint32 [n_tasks] (-1 = none)
    best_filled_ns: torch.Tensor      # int64 [n_tasks]


def fikit_pairing_workspace_bytes(n_tasks: int) -> int:
    return int(load().fikit_pairing_workspace_bytes(n_tasks))


def fikit_pairing_best(hp_task: torch.Tensor, lp_task: torch.Tensor, n_tasks: int, gap_offsets: torch.Tensor,
                       filled_ns: torch.Tensor, lp_completion_ns: torch.Tensor, *, out: Optional[Pairing] = None,
                       workspace_buf: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> Pairing:
    """hp_task, lp_task: int32 [S]; gap_offsets: int64 [S+1]; filled_ns: int64 [n_gaps]; lp_completion_ns: int64 [S]."""
    lib = load()
    dev = hp_task.device
    s = hp_task.numel()
    assert hp_task.dtype == torch.int32 and lp_task.dtype == torch.int32 and lp_task.numel() == s
    assert gap_offsets.dtype == torch.int64 and gap_offsets.numel() == s + 1
    assert filled_ns.dtype == torch.int64 and lp_completion_ns.dtype == torch.int64 and lp_completion_ns.numel() == s
    for t in (hp_task, lp_task, gap_offsets, filled_ns, lp_completion_ns):
        assert t.is_contiguous() and t.device == dev
    if out is None:
        out = Pairing(torch.empty(s, dtype=torch.int64, device=dev), torch.empty(n_tasks, dtype=torch.int64, device=dev),
                      torch.empty(n_tasks, dtype=torch.int32, device=dev), torch.empty(n_tasks, dtype=torch.int64, device=dev))
    if workspace_buf is None:
        workspace_buf = workspace(fikit_pairing_workspace_bytes(n_tasks), dev)
    with torch.cuda.device(dev):
        st = lib.fikit_pairing_best(_ptr(hp_task), _ptr(lp_task), s, n_tasks, _ptr(gap_offsets), _ptr(filled_ns),
                                    _ptr(lp_completion_ns), _ptr(out.scenario_filled_ns), _ptr(out.best_scenario),
                                    _ptr(out.best_lp), _ptr(out.best_filled_ns), _ptr(workspace_buf), workspace_buf.numel(),
                                    _stream_handle(stream))
    if st != FIKIT_OK:
        raise FikitError(st, "fikit_pairing_best")
    return out


class MergedProfile(NamedTuple):
    rows: torch.Tensor              # uint8 [n_rows, 128]
    task_row_offsets: torch.Tensor  # int64 [n_tasks + 1]
    n_rows: int


def fikit_profile_merge_workspace_bytes(n_tasks: int) -> int:
    return int(load().fikit_profile_merge_workspace_bytes(n_tasks))


def fikit_profile_merge(rows_a: torch.Tensor, task_row_offsets_a: torch.Tensor, rows_b: torch.Tensor,
                        task_row_offsets_b: torch.Tensor, *, row_capacity: Optional[int] = None,
                        rows_out: Optional[torch.Tensor] = None, task_row_offsets_out: Optional[torch.Tensor] = None,
                        workspace_buf: Optional[torch.Tensor] = None,
                        stream: Optional[torch.cuda.Stream] = None) -> MergedProfile:
    """rows_*: uint8 [n, 128] (fikit_profile's rows); task_row_offsets_*: int64 [n_tasks + 1]."""
    lib = load()
    dev = task_row_offsets_a.device
    n_tasks = task_row_offsets_a.numel() - 1
    assert task_row_offsets_b.numel() == n_tasks + 1
    assert task_row_offsets_a.dtype == torch.int64 and task_row_offsets_b.dtype == torch.int64
    for t in (rows_a, rows_b):
        assert t.dtype == torch.uint8 and t.is_contiguous() and t.device == dev and t.numel() % ROW_BYTES == 0
    if row_capacity is None:
        row_capacity = rows_out.shape[0] if rows_out is not None else (rows_a.numel() + rows_b.numel()) // ROW_BYTES
    if rows_out is None:
        rows_out = torch.empty((row_capacity, ROW_BYTES), dtype=torch.uint8, device=dev)
    if task_row_offsets_out is None:
        task_row_offsets_out = torch.empty(n_tasks + 1, dtype=torch.int64, device=dev)
    if workspace_buf is None:
        workspace_buf = workspace(fikit_profile_merge_workspace_bytes(n_tasks), dev)
    n_rows = ctypes.c_uint64(0)
    with torch.cuda.device(dev):
        st = lib.fikit_profile_merge(_ptr(rows_a), _ptr(task_row_offsets_a), _ptr(rows_b), _ptr(task_row_offsets_b), n_tasks,
                                     _ptr(rows_out), row_capacity, _ptr(task_row_offsets_out), ctypes.byref(n_rows),
                                     _ptr(workspace_buf), workspace_buf.numel(), _stream_handle(stream))
    if st != FIKIT_OK:
        raise FikitError(st, "fikit_profile_merge", n_rows=n_rows.value)
    return MergedProfile(rows_out[: n_rows.value], task_row_offsets_out, n_rows.value)


# ---- helpers to move host arrays in and out (marshalling only) ---------------------------------
def to_device_records(records: np.ndarray, device) -> torch.Tensor:
    assert records.dtype.itemsize == LAUNCH_BYTES
    flat = np.ascontiguousarray(records).view(np.uint8).reshape(-1, LAUNCH_BYTES)
    return torch.from_numpy(flat).to(device)


def to_device_u64(a: np.ndarray, device) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint64).view(np.int64)).to(device)


def to_device_u32(a: np.ndarray, device) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint32).view(np.int32)).to(device)


def rows_to_numpy(rows: torch.Tensor) -> np.ndarray:
    return rows.cpu().numpy().reshape(-1).view(ROW_DTYPE).copy()


def u64_to_numpy(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)


def u32_to_numpy(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)
