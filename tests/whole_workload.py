"""Whole-workload comparison of the HIP library's outputs with the CPU oracle at full size.

The library's outputs are copied into shared host memory; worker processes then regenerate the
workload piece by piece from its seeds (ranges of whole tasks, for the batched workload whole
scenarios), run the single-threaded oracle on each piece and compare every element of that piece:
Kernel IDs, rows and row offsets, and for scenarios the per-gap fill counts and filled times, the
completion time and the number of kernels placed.  Only verdicts travel back.

Workers are started through the fork server (which conftest.py starts before any test touches the
GPU) and never use the GPU themselves.
"""
from __future__ import annotations

import time
from multiprocessing import shared_memory
from typing import Dict, Optional

import numpy as np


class SharedArrays:
    """Named host arrays in shared memory (created by the test, attached by the workers)."""

    def __init__(self):
        self._blocks = []
        self.spec: Dict[str, tuple] = {}      # name -> (shm name, dtype string, length)
        self.views: Dict[str, np.ndarray] = {}

    def put(self, name: str, dtype, length: int) -> np.ndarray:
        dt = np.dtype(dtype)
        shm = shared_memory.SharedMemory(create=True, size=max(1, length * dt.itemsize))
        self._blocks.append(shm)
        view = np.ndarray((length,), dtype=dt, buffer=shm.buf)
        self.spec[name] = (shm.name, dt.str if dt.names is None else "rows", length)
        self.views[name] = view
        return view

    def close(self):
        self.views.clear()
        for shm in self._blocks:
            shm.close()
            shm.unlink()
        self._blocks = []


def _attach(spec):
    import oracle
    blocks, views = [], {}
    for name, (shm_name, dt, length) in spec.items():
        shm = shared_memory.SharedMemory(name=shm_name)
        blocks.append(shm)
        dtype = oracle.ROW_DTYPE if dt == "rows" else np.dtype(dt)
        views[name] = np.ndarray((length,), dtype=dtype, buffer=shm.buf)
    return blocks, views


def _first_diff(a: np.ndarray, b: np.ndarray) -> int:
    if a.shape != b.shape:
        return -1
    if a.dtype.names is not None:
        a = a.view(np.uint64).reshape(a.shape[0], -1)
        b = b.view(np.uint64).reshape(b.shape[0], -1)
        bad = np.nonzero((a != b).any(axis=1))[0]
    else:
        bad = np.nonzero(a != b)[0]
    return int(bad[0]) if bad.size else -2


def check_piece(args):
    """Worker: tasks [t_lo, t_hi) of the workload against the library's outputs in shared memory.
    -> dict(tasks, scenarios, equal_tasks, equal_scenarios, errors[list of str], seconds)."""
    import oracle
    from paper_2311_10359_amd import traces
    index, overrides, t_lo, t_hi, spec, with_scenarios = args
    t0 = time.time()
    cfg = traces.config(index, **dict(overrides))
    blocks, g = _attach(spec)
    errors = []
    try:
        tasks = range(t_lo, t_hi)
        rec, off = traces.build(cfg, tasks=tasks)
        o_ids, o_rows, o_tro = oracle.profile(rec, off)
        del rec
        goff = g["task_offsets"]
        first = int(goff[t_lo])
        assert int(goff[t_hi]) - first == int(off[-1])
        d = _first_diff(g["ids"][first:first + o_ids.shape[0]], o_ids)
        if d != -2:
            errors.append(f"tasks {t_lo}..{t_hi - 1}: Kernel IDs differ first at launch {first + d}")
        tro = g["task_row_offsets"]
        r_lo, r_hi = int(tro[t_lo]), int(tro[t_hi])
        if not np.array_equal(tro[t_lo:t_hi + 1] - tro[t_lo], o_tro):
            errors.append(f"tasks {t_lo}..{t_hi - 1}: row offsets differ")
        expect = o_rows.copy()
        expect["task"] += np.uint32(t_lo)
        d = _first_diff(g["rows"][r_lo:r_hi], expect)
        if d != -2:
            errors.append(f"tasks {t_lo}..{t_hi - 1}: rows differ (first at row {r_lo + d}; -1: count {r_hi - r_lo} vs {expect.shape[0]})")
        n_scen = 0
        if with_scenarios:
            # scenario s = (task 2s, task 2s + 1); a piece holds whole scenarios
            assert t_lo % 2 == 0 and t_hi % 2 == 0
            s_lo, s_hi = t_lo // 2, t_hi // 2
            n_scen = s_hi - s_lo
            hp = np.arange(0, t_hi - t_lo, 2, dtype=np.uint32)
            lp = hp + 1
            go = traces.gap_offsets(off, hp)
            fc, fn, comp, placed = oracle.gapfill(o_ids, off, o_rows, o_tro, hp, lp, cfg.margin_ns, cfg.min_gap_ns, go)
            ggo = g["gap_offsets"]
            g_lo, g_hi = int(ggo[s_lo]), int(ggo[s_hi])
            if not np.array_equal(ggo[s_lo:s_hi + 1] - ggo[s_lo], go):
                errors.append(f"scenarios {s_lo}..{s_hi - 1}: gap offsets differ")
            for name, exp, lo, hi in (("fill_count", fc, g_lo, g_hi), ("filled_ns", fn, g_lo, g_hi),
                                      ("lp_completion_ns", comp, s_lo, s_hi), ("lp_placed", placed, s_lo, s_hi)):
                d = _first_diff(g[name][lo:hi], exp)
                if d != -2:
                    errors.append(f"scenarios {s_lo}..{s_hi - 1}: {name} differs first at {lo + d}")
        ok = not errors
        return {"tasks": t_hi - t_lo, "scenarios": n_scen, "equal_tasks": (t_hi - t_lo) if ok else 0,
                "equal_scenarios": n_scen if ok else 0, "errors": errors, "seconds": time.time() - t0}
    finally:
        del g
        for shm in blocks:
            shm.close()


def compare_whole_workload(cfg, off: np.ndarray, outputs: Dict[str, "object"], *, records_per_piece: int = 4 << 20,
                           workers: int = 16, say=print) -> dict:
    """outputs: torch device tensors by name: ids, rows (uint8 [R, 128]), task_row_offsets and, for workloads with
    scenarios, gap_offsets, fill_count, filled_ns, lp_completion_ns, lp_placed.  Every element is compared; returns
    the totals.  Raises AssertionError naming the first differences."""
    import multiprocessing as mp
    from concurrent.futures import ProcessPoolExecutor, as_completed

    import torch

    import oracle
    with_scenarios = "fill_count" in outputs
    sh = SharedArrays()
    t0 = time.time()
    try:
        host_types = {"ids": np.uint64, "task_row_offsets": np.uint64, "gap_offsets": np.uint64, "fill_count": np.uint32,
                      "filled_ns": np.int64, "lp_completion_ns": np.int64, "lp_placed": np.uint64}
        sh.put("task_offsets", np.uint64, off.shape[0])[:] = off
        for name, t in outputs.items():
            if name == "rows":
                view = sh.put(name, oracle.ROW_DTYPE, t.shape[0])
                dst = torch.from_numpy(view.view(np.uint8).reshape(-1, 128))
            else:
                view = sh.put(name, host_types[name], t.numel())
                signed = {np.uint64: np.int64, np.uint32: np.int32}.get(host_types[name], host_types[name])
                dst = torch.from_numpy(view.view(signed))
            dst.copy_(t)
        if torch.cuda.is_available():
            torch.cuda.synchronize()
        say(f"  outputs copied to the host in {time.time() - t0:.1f}s")
        # pieces of whole tasks (an even number of them where tasks pair up into scenarios)
        pieces = []
        lo = 0
        step = 2 if with_scenarios else 1
        while lo < cfg.n_tasks:
            hi = lo + step
            while hi < cfg.n_tasks and int(off[min(hi + step, cfg.n_tasks)] - off[lo]) <= records_per_piece:
                hi += step
            hi = min(hi, cfg.n_tasks)
            pieces.append((lo, hi))
            lo = hi
        total = {"tasks": 0, "scenarios": 0, "equal_tasks": 0, "equal_scenarios": 0, "errors": [], "cpu_seconds": 0.0}
        ctx = mp.get_context("forkserver")
        last = time.time()
        with ProcessPoolExecutor(max_workers=workers, mp_context=ctx) as pool:
            futs = [pool.submit(check_piece, (cfg.index, cfg.overrides, a, b, sh.spec, with_scenarios)) for a, b in pieces]
            done = 0
            for f in as_completed(futs):
                r = f.result()
                done += 1
                for k in ("tasks", "scenarios", "equal_tasks", "equal_scenarios"):
                    total[k] += r[k]
                total["errors"] += r["errors"]
                total["cpu_seconds"] += r["seconds"]
                if time.time() - last > 15:
                    last = time.time()
                    say(f"  oracle pieces {done}/{len(pieces)} ({time.time() - t0:.0f}s)")
        total["wall_seconds"] = time.time() - t0
        msg = f"  {total['equal_tasks']}/{total['tasks']} tasks"
        if with_scenarios:
            msg += f", {total['equal_scenarios']}/{total['scenarios']} scenarios"
        say(msg + f" equal ({len(pieces)} pieces, {total['cpu_seconds']:.0f} s of oracle and generator time on {workers} processes, "
                  f"{total['wall_seconds']:.1f}s wall)")
        assert not total["errors"], "; ".join(total["errors"][:5])
        assert total["tasks"] == cfg.n_tasks and total["equal_tasks"] == cfg.n_tasks
        return total
    finally:
        sh.close()
