"""CPU oracle (test infrastructure only).

The C++ source `fikit_oracle.cpp` is the definition of correct output for the trace-profiling
and gap-filling path; this package compiles it with g++ and wraps it with ctypes.  It is
imported by the tests, by the smoke check and by the benchmark's CPU-baseline leg, never by
the product, and it imports nothing from the product.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fikit_oracle.cpp")
_LIB = os.path.join(_HERE, "libfikit_oracle.so")

# Own description of the two record layouts (not shared with the product).
STATS_DTYPE = np.dtype([("count", "<u8"), ("sum", "<u8"), ("min", "<i8"), ("max", "<i8"),
                        ("p50", "<i8"), ("p95", "<i8")])
ROW_DTYPE = np.dtype([("kernel_id", "<u8"), ("task", "<u4"), ("reserved0", "<u4"),
                      ("exec", STATS_DTYPE), ("gap", STATS_DTYPE), ("reserved1", "u1", (16,))])
assert STATS_DTYPE.itemsize == 48 and ROW_DTYPE.itemsize == 128

OK, INVALID_ARG, ROW_CAPACITY, BAD_RECORD, UNKNOWN_ID = 0, -1, -3, -4, -5


class OracleError(RuntimeError):
    def __init__(self, status: int):
        super().__init__(f"oracle status {status}")
        self.status = status


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (plain -O2, no threads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, u64, u32, i64 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int64
        lib.oracle_kernel_id.restype = u64
        lib.oracle_kernel_id.argtypes = [vp, u64]
        lib.oracle_profile.restype = ctypes.c_int
        lib.oracle_profile.argtypes = [vp, u64, vp, u32, vp, vp, u64, vp, vp]
        lib.oracle_gapfill.restype = ctypes.c_int
        lib.oracle_gapfill.argtypes = [vp, vp, u32, vp, vp, vp, vp, u64, i64, i64, vp, vp, vp, vp,
                                       vp, vp, vp, ctypes.c_int]
        lib.oracle_measure.restype = ctypes.c_int
        lib.oracle_measure.argtypes = [vp, u64, vp, u32, vp, vp]
        lib.oracle_replay.restype = ctypes.c_int
        lib.oracle_replay.argtypes = [vp, vp, u32, vp, vp, vp, vp, vp, u64, i64, i64, ctypes.c_int, vp, vp, vp,
                                      vp, vp, ctypes.c_int]
        lib.oracle_profile_merge.restype = ctypes.c_int
        lib.oracle_profile_merge.argtypes = [vp, vp, vp, vp, u32, vp, u64, vp, vp]
        lib.oracle_pairing_best.restype = ctypes.c_int
        lib.oracle_pairing_best.argtypes = [vp, vp, u64, u32, vp, vp, vp, vp, vp, vp, vp]
        lib.oracle_prio_fill.restype = ctypes.c_int
        lib.oracle_prio_fill.argtypes = [vp, vp, u32, vp, vp, vp, vp, vp, vp, u64, i64, i64, ctypes.c_int, vp, vp, vp,
                                         vp, vp, vp, vp]
        _lib = lib
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


def kernel_id(data: bytes) -> int:
    buf = np.frombuffer(data, dtype=np.uint8) if len(data) else np.zeros(0, dtype=np.uint8)
    return int(_load().oracle_kernel_id(_p(np.ascontiguousarray(buf)), len(data)))


def profile(records: np.ndarray, task_offsets: np.ndarray, row_capacity: Optional[int] = None
            ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """-> (ids[n], rows[R], task_row_offsets[T+1]).  Raises OracleError on a non-zero status."""
    assert records.dtype.itemsize == 64
    records = np.ascontiguousarray(records)
    task_offsets = np.ascontiguousarray(task_offsets, dtype=np.uint64)
    n = records.shape[0]
    n_tasks = task_offsets.shape[0] - 1
    cap = n if row_capacity is None else row_capacity
    ids = np.zeros(n, dtype=np.uint64)
    rows = np.zeros(cap, dtype=ROW_DTYPE)
    tro = np.zeros(n_tasks + 1, dtype=np.uint64)
    n_rows = np.zeros(1, dtype=np.uint64)
    st = _load().oracle_profile(_p(records), n, _p(task_offsets), n_tasks, _p(ids), _p(rows), cap,
                                _p(tro), _p(n_rows))
    if st != OK:
        err = OracleError(st)
        err.n_rows = int(n_rows[0])
        raise err
    return ids, rows[: int(n_rows[0])].copy(), tro


def gapfill(ids: np.ndarray, task_offsets: np.ndarray, rows: np.ndarray, task_row_offsets: np.ndarray,
            hp_task: np.ndarray, lp_task: np.ndarray, margin_ns: int, min_gap_ns: int,
            gap_offsets: np.ndarray, want_assign: bool = False, predictor: int = 0):
    """-> (fill_count, filled_ns, lp_completion_ns, lp_placed[, assign, assign_offsets]).
    predictor: 0 = nearest-rank median of the ID's samples, 1 = their mean (sum // count)."""
    ids = np.ascontiguousarray(ids, dtype=np.uint64)
    task_offsets = np.ascontiguousarray(task_offsets, dtype=np.uint64)
    rows = np.ascontiguousarray(rows)
    assert rows.dtype.itemsize == 128
    tro = np.ascontiguousarray(task_row_offsets, dtype=np.uint64)
    hp = np.ascontiguousarray(hp_task, dtype=np.uint32)
    lp = np.ascontiguousarray(lp_task, dtype=np.uint32)
    go = np.ascontiguousarray(gap_offsets, dtype=np.uint64)
    s = hp.shape[0]
    n_tasks = task_offsets.shape[0] - 1
    n_gaps = int(go[-1]) if s else 0
    fill_count = np.zeros(n_gaps, dtype=np.uint32)
    filled_ns = np.zeros(n_gaps, dtype=np.int64)
    completion = np.zeros(s, dtype=np.int64)
    placed = np.zeros(s, dtype=np.uint64)
    assign = assign_off = None
    if want_assign:
        lens = (task_offsets[1:] - task_offsets[:-1])[lp.astype(np.int64)] if s else np.zeros(0, np.uint64)
        assign_off = np.zeros(s + 1, dtype=np.uint64)
        np.cumsum(lens, out=assign_off[1:])
        assign = np.zeros(int(assign_off[-1]), dtype=np.uint32)
    st = _load().oracle_gapfill(_p(ids), _p(task_offsets), n_tasks, _p(rows), _p(tro), _p(hp), _p(lp),
                                s, margin_ns, min_gap_ns, _p(go), _p(fill_count), _p(filled_ns),
                                _p(completion), _p(placed), _p(assign_off), _p(assign), predictor)
    if st != OK:
        raise OracleError(st)
    if want_assign:
        return fill_count, filled_ns, completion, placed, assign, assign_off
    return fill_count, filled_ns, completion, placed


def measure(records: np.ndarray, task_offsets: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """-> (exec_ns[n], gap_ns[n]); gap_ns is -1 for the last launch of a task."""
    assert records.dtype.itemsize == 64
    records = np.ascontiguousarray(records)
    task_offsets = np.ascontiguousarray(task_offsets, dtype=np.uint64)
    n = records.shape[0]
    ex = np.zeros(n, dtype=np.int64)
    gp = np.zeros(n, dtype=np.int64)
    st = _load().oracle_measure(_p(records), n, _p(task_offsets), task_offsets.shape[0] - 1, _p(ex), _p(gp))
    if st != OK:
        raise OracleError(st)
    return ex, gp


def replay(ids: np.ndarray, task_offsets: np.ndarray, rows: np.ndarray, task_row_offsets: np.ndarray,
           actual_gap_ns: np.ndarray, hp_task: np.ndarray, lp_task: np.ndarray, margin_ns: int, min_gap_ns: int,
           feedback: bool, gap_offsets: np.ndarray, predictor: int = 0):
    """-> (fill_count, filled_ns, hp_delay_ns, lp_placed)."""
    ids = np.ascontiguousarray(ids, dtype=np.uint64)
    task_offsets = np.ascontiguousarray(task_offsets, dtype=np.uint64)
    rows = np.ascontiguousarray(rows)
    assert rows.dtype.itemsize == 128
    tro = np.ascontiguousarray(task_row_offsets, dtype=np.uint64)
    ag = np.ascontiguousarray(actual_gap_ns, dtype=np.int64)
    hp = np.ascontiguousarray(hp_task, dtype=np.uint32)
    lp = np.ascontiguousarray(lp_task, dtype=np.uint32)
    go = np.ascontiguousarray(gap_offsets, dtype=np.uint64)
    s = hp.shape[0]
    n_gaps = int(go[-1]) if s else 0
    fill_count = np.zeros(n_gaps, dtype=np.uint32)
    filled_ns = np.zeros(n_gaps, dtype=np.int64)
    delay = np.zeros(s, dtype=np.int64)
    placed = np.zeros(s, dtype=np.uint64)
    st = _load().oracle_replay(_p(ids), _p(task_offsets), task_offsets.shape[0] - 1, _p(rows), _p(tro), _p(ag),
                               _p(hp), _p(lp), s, margin_ns, min_gap_ns, 1 if feedback else 0, _p(go),
                               _p(fill_count), _p(filled_ns), _p(delay), _p(placed), predictor)
    if st != OK:
        raise OracleError(st)
    return fill_count, filled_ns, delay, placed


def prio_fill(ids: np.ndarray, task_offsets: np.ndarray, rows: np.ndarray, task_row_offsets: np.ndarray,
              hp_task: np.ndarray, lp_offsets: np.ndarray, lp_task: np.ndarray, lp_prio: np.ndarray, margin_ns: int,
              min_gap_ns: int, gap_offsets: np.ndarray, predictor: int = 0, want_issue: bool = False):
    """Several low-priority tasks per scenario (entries lp_offsets[s]..lp_offsets[s+1] of lp_task / lp_prio).
    -> (fill_count, filled_ns, lp_placed[entries], lp_placed_ns[entries][, issue_entry, issue_offsets])."""
    ids = np.ascontiguousarray(ids, dtype=np.uint64)
    task_offsets = np.ascontiguousarray(task_offsets, dtype=np.uint64)
    rows = np.ascontiguousarray(rows)
    assert rows.dtype.itemsize == 128
    tro = np.ascontiguousarray(task_row_offsets, dtype=np.uint64)
    hp = np.ascontiguousarray(hp_task, dtype=np.uint32)
    lo = np.ascontiguousarray(lp_offsets, dtype=np.uint64)
    lt = np.ascontiguousarray(lp_task, dtype=np.uint32)
    lq = np.ascontiguousarray(lp_prio, dtype=np.uint32)
    go = np.ascontiguousarray(gap_offsets, dtype=np.uint64)
    s = hp.shape[0]
    assert lo.shape[0] == s + 1 and lt.shape[0] == lq.shape[0]
    n_gaps = int(go[-1]) if s else 0
    n_entries = lt.shape[0]
    fill_count = np.zeros(n_gaps, dtype=np.uint32)
    filled_ns = np.zeros(n_gaps, dtype=np.int64)
    placed = np.zeros(n_entries, dtype=np.uint64)
    placed_ns = np.zeros(n_entries, dtype=np.int64)
    issue = issue_off = None
    if want_issue:
        lens = (task_offsets[1:] - task_offsets[:-1])[lt.astype(np.int64)] if n_entries else np.zeros(0, np.uint64)
        per_scen = np.zeros(s, dtype=np.uint64)
        for k in range(s):
            per_scen[k] = lens[int(lo[k]):int(lo[k + 1])].sum()
        issue_off = np.zeros(s + 1, dtype=np.uint64)
        np.cumsum(per_scen, out=issue_off[1:])
        issue = np.full(int(issue_off[-1]), 0xffffffff, dtype=np.uint32)
    st = _load().oracle_prio_fill(_p(ids), _p(task_offsets), task_offsets.shape[0] - 1, _p(rows), _p(tro), _p(hp), _p(lo),
                                  _p(lt), _p(lq), s, margin_ns, min_gap_ns, predictor, _p(go), _p(fill_count),
                                  _p(filled_ns), _p(placed), _p(placed_ns), _p(issue_off), _p(issue))
    if st != OK:
        raise OracleError(st)
    if want_issue:
        return fill_count, filled_ns, placed, placed_ns, issue, issue_off
    return fill_count, filled_ns, placed, placed_ns


def pairing_best(hp_task: np.ndarray, lp_task: np.ndarray, n_tasks: int, gap_offsets: np.ndarray, filled_ns: np.ndarray,
                 lp_completion_ns: np.ndarray):
    """-> (scenario_filled_ns[S], best_scenario[n_tasks], best_lp[n_tasks], best_filled_ns[n_tasks])."""
    hp = np.ascontiguousarray(hp_task, dtype=np.uint32)
    lp = np.ascontiguousarray(lp_task, dtype=np.uint32)
    go = np.ascontiguousarray(gap_offsets, dtype=np.uint64)
    fn = np.ascontiguousarray(filled_ns, dtype=np.int64)
    comp = np.ascontiguousarray(lp_completion_ns, dtype=np.int64)
    s = hp.shape[0]
    assert lp.shape[0] == s and go.shape[0] == s + 1 and comp.shape[0] == s
    assert s == 0 or fn.shape[0] >= int(go[-1])
    total = np.zeros(s, dtype=np.int64)
    best_s = np.zeros(n_tasks, dtype=np.uint64)
    best_lp = np.zeros(n_tasks, dtype=np.uint32)
    best_f = np.zeros(n_tasks, dtype=np.int64)
    st = _load().oracle_pairing_best(_p(hp), _p(lp), s, n_tasks, _p(go), _p(fn), _p(comp), _p(total), _p(best_s),
                                     _p(best_lp), _p(best_f))
    if st != OK:
        raise OracleError(st)
    return total, best_s, best_lp, best_f


def profile_merge(a_rows: np.ndarray, a_offsets: np.ndarray, b_rows: np.ndarray, b_offsets: np.ndarray,
                  row_capacity: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """-> (rows[n_rows], task_row_offsets[n_tasks + 1]) of the merged profile."""
    a_rows = np.ascontiguousarray(a_rows)
    b_rows = np.ascontiguousarray(b_rows)
    assert a_rows.dtype.itemsize == 128 and b_rows.dtype.itemsize == 128
    ao = np.ascontiguousarray(a_offsets, dtype=np.uint64)
    bo = np.ascontiguousarray(b_offsets, dtype=np.uint64)
    assert ao.shape == bo.shape
    n_tasks = ao.shape[0] - 1
    cap = a_rows.shape[0] + b_rows.shape[0] if row_capacity is None else row_capacity
    out = np.zeros(cap, dtype=a_rows.dtype)
    oo = np.zeros(n_tasks + 1, dtype=np.uint64)
    n = ctypes.c_uint64(0)
    st = _load().oracle_profile_merge(_p(a_rows), _p(ao), _p(b_rows), _p(bo), n_tasks, _p(out), cap, _p(oo), ctypes.byref(n))
    if st != OK:
        err = OracleError(st)
        err.n_rows = n.value
        raise err
    return out[: n.value].copy(), oo
