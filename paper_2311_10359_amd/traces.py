"""Seeded synthetic kernel-launch traces.

Stands in for the output of the paper's measurement phase (Section 3.2, "Measuring the
execution and idle time of kernel"): per task, the sequence of intercepted kernel launches,
each with the ingredients of its Kernel ID (function name, grid and block dimensions; plus
dynamic shared-memory bytes) and the device start and end time of the kernel.

This module only *draws inputs*.  It contains none of the method's arithmetic (no hashing,
no statistics, no schedule evaluation) so that the CPU oracle and the HIP library can both be
fed from it without sharing anything else.

The five workloads mirror the structure the paper describes: a service re-executes the same
kernel sequence again and again (Section 3.2), few distinct Kernel IDs recur within and
across runs, the same ID shows somewhat different durations from launch to launch, and idle
gaps come from launch overhead with occasional long host-side stalls (Section 1).

Every task has its own counter-seeded generator, so any single task can be regenerated alone
(used by the sampled full-size parity checks).
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Callable, Optional, Sequence, Tuple

import numpy as np

# One launch record: 64 bytes, little endian.
LAUNCH_DTYPE = np.dtype(
    [
        ("name_id", "<u4"),
        ("grid", "<u4", (3,)),
        ("block", "<u4", (3,)),
        ("shmem", "<u4"),
        ("start_ns", "<i8"),
        ("end_ns", "<i8"),
        ("run", "<u4"),
        ("reserved", "u1", (12,)),
    ]
)
assert LAUNCH_DTYPE.itemsize == 64

BASE_SEED = 2311

# Share of the log-scale variance that belongs to the Kernel ID (the kernel's characteristic
# duration) rather than to the individual launch.  The marginal over launches stays exactly
# lognormal(mu, sigma) because rho^2 + (1 - rho^2) = 1.
RHO_EXEC = 0.95
RHO_GAP = 0.90


@dataclass(frozen=True)
class TraceConfig:
    index: int
    name: str
    n_tasks: int
    # launches(task) -> number of launches, ids(task) -> number of distinct kernel tuples
    launches: Callable[[int], int]
    ids: Callable[[int], int]
    pattern: str  # "pass50" | "pass200x2" | "zipf" | "uniform" | "pass2k"
    exec_mu: Callable[[int], float]
    exec_sigma: Callable[[int], float]
    gap_mu: Callable[[int], float]
    gap_sigma: Callable[[int], float]
    stall_frac: float = 0.0  # share of gaps drawn from the stall distribution
    stall_mu: float = 0.0
    stall_sigma: float = 0.0
    zero_gap_frac: float = 0.0  # share of gaps that are exactly 0 (back-to-back launches)
    zipf_s: float = 0.0
    scenario_kind: str = "none"  # "pair01" | "grid" | "adjacent" | "none"
    margin_ns: int = 500
    min_gap_ns: int = 0
    runs: int = 1  # measured runs per task: the trace is cut into this many runs of (almost) equal length
    rho_exec: float = RHO_EXEC  # share of the log-scale spread of execution times that belongs to the Kernel ID
    rho_gap: float = RHO_GAP    # the same for idle times (0 for both: every launch drawn independently)
    overrides: tuple = ()  # the keyword overrides config() was called with (to rebuild it elsewhere)

    @property
    def n_records(self) -> int:
        return sum(self.launches(t) for t in range(self.n_tasks))


def _const(v):
    return lambda task: v


def config(index: int, *, n_tasks: Optional[int] = None, launches: Optional[int] = None,
           hp_launches: Optional[int] = None, lp_launches: Optional[int] = None, runs: Optional[int] = None,
           rho: Optional[float] = None) -> TraceConfig:
    """The five workloads.  Keyword overrides shrink a workload while keeping its structure
    (same distributions, same ID pattern) so that it can be checked on a CPU in seconds."""
    ln = math.log
    if index == 0:
        n = launches or 1000
        cfg = TraceConfig(
            0, "tiny", 2, _const(n), lambda t: 20 if t == 0 else 15, "pass50",
            _const(ln(20000)), _const(0.8), _const(ln(8000)), _const(1.0),
            scenario_kind="pair01")
    elif index == 1:
        n = launches or 65536
        cfg = TraceConfig(
            1, "medium", n_tasks or 32, _const(n), _const(300), "pass200x2",
            _const(ln(20000)), _const(0.8), _const(ln(8000)), _const(1.0),
            stall_frac=0.10, stall_mu=ln(200000), stall_sigma=0.5, scenario_kind="grid")
    elif index == 2:
        n = launches or 1048576
        cfg = TraceConfig(
            2, "skewed", n_tasks or 64, _const(n), _const(4096), "zipf",
            _const(ln(5000)), _const(1.5), _const(ln(15000)), _const(1.2),
            zero_gap_frac=0.30, zipf_s=1.2)
    elif index == 3:
        n = launches or 1048576
        cfg = TraceConfig(
            3, "large_profile", n_tasks or 256, _const(n), _const(1000), "uniform",
            _const(ln(20000)), _const(0.8), _const(ln(8000)), _const(1.0))
    elif index == 4:
        h = hp_launches or 4096
        l = lp_launches or 16384
        nt = n_tasks or 131072
        assert nt % 2 == 0
        # even task = high-priority trace, odd task = low-priority queue of the same scenario
        cfg = TraceConfig(
            4, "batched_gapfill", nt,
            lambda t: h if t % 2 == 0 else l,
            lambda t: 100 if t % 2 == 0 else 80, "pass2k",
            lambda t: ln(20000) if t % 2 == 0 else ln(6000),
            lambda t: 0.8 if t % 2 == 0 else 1.0,
            lambda t: ln(30000) if t % 2 == 0 else ln(8000),
            lambda t: 1.2 if t % 2 == 0 else 1.0,
            scenario_kind="adjacent")
    else:
        raise ValueError(f"no workload {index}")
    ov = tuple((k, v) for k, v in (("n_tasks", n_tasks), ("launches", launches), ("hp_launches", hp_launches),
                                   ("lp_launches", lp_launches), ("runs", runs), ("rho", rho)) if v is not None)
    cfg = replace(cfg, overrides=ov, runs=runs or 1)
    if rho is not None:
        # rho scales both shares: 1 keeps the defaults, 0 draws every launch independently of its Kernel ID
        cfg = replace(cfg, rho_exec=RHO_EXEC * rho, rho_gap=RHO_GAP * rho)
    return cfg


def _rng(cfg: TraceConfig, task: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([BASE_SEED + cfg.index, task, stream]))


def kernel_tuples(cfg: TraceConfig, task: int) -> np.ndarray:
    """K distinct (name_id, grid[3], block[3], shmem) tuples of a task as a (K, 8) uint32 array."""
    k = cfg.ids(task)
    rng = _rng(cfg, task, 0)
    out = np.zeros((0, 8), dtype=np.uint32)
    grid_y_choices = np.array([1, 1, 1, 2, 4, 8, 16, 32, 64], dtype=np.uint32)
    block_x_choices = np.array([32, 64, 128, 256, 512, 1024], dtype=np.uint32)
    block_y_choices = np.array([1, 1, 2, 4], dtype=np.uint32)
    while out.shape[0] < k:
        m = k - out.shape[0] + 8
        t = np.zeros((m, 8), dtype=np.uint32)
        t[:, 0] = rng.integers(0, 1 << 20, m)
        t[:, 1] = rng.integers(1, 65536, m)
        t[:, 2] = rng.choice(grid_y_choices, m)
        t[:, 3] = 1
        bx = rng.choice(block_x_choices, m)
        by = rng.choice(block_y_choices, m)
        by = np.where(bx.astype(np.uint64) * by > 1024, 1, by).astype(np.uint32)
        t[:, 4] = bx
        t[:, 5] = by
        t[:, 6] = 1
        sh = rng.integers(1, 257, m).astype(np.uint32) * 256
        t[:, 7] = np.where(rng.random(m) < 0.5, 0, sh)
        out = np.concatenate([out, t], axis=0)
        # keep the first occurrence of each (name_id, grid.x) pair, in draw order
        key = (out[:, 0].astype(np.uint64) << np.uint64(16)) | out[:, 1].astype(np.uint64)
        _, first = np.unique(key, return_index=True)
        out = out[np.sort(first)]
    return out[:k]


def _id_sequence(cfg: TraceConfig, task: int, n: int, k: int) -> np.ndarray:
    """Index (0..k-1) of the kernel tuple used by each of the n launches."""
    rng = _rng(cfg, task, 1)
    if cfg.pattern == "pass50":
        plen = max(50, k)
        one = np.concatenate([np.arange(k), rng.integers(0, k, plen - k)])
        rng.shuffle(one)
        reps = -(-n // plen)
        return np.tile(one, reps)[:n]
    if cfg.pattern == "pass200x2":
        # two variants of the model pass that together touch all k tuples
        plen = (2 * k) // 3
        a = rng.permutation(plen)
        b = rng.permutation(plen) + (k - plen)
        reps = -(-n // plen)
        pick = rng.random(reps) < 0.5
        seq = np.where(pick[:, None], a[None, :], b[None, :]).reshape(-1)
        return seq[:n]
    if cfg.pattern == "zipf":
        w = 1.0 / np.power(np.arange(1, k + 1, dtype=np.float64), cfg.zipf_s)
        cdf = np.cumsum(w / w.sum())
        cdf[-1] = 1.0
        return np.searchsorted(cdf, rng.random(n), side="right").clip(0, k - 1)
    if cfg.pattern == "uniform":
        return rng.integers(0, k, n)
    if cfg.pattern == "pass2k":
        one = np.concatenate([np.arange(k), np.arange(k)])
        rng.shuffle(one)
        reps = -(-n // one.size)
        return np.tile(one, reps)[:n]
    raise ValueError(cfg.pattern)


def task_records(cfg: TraceConfig, task: int, out: Optional[np.ndarray] = None) -> np.ndarray:
    """All launch records of one task, in launch order.  `out`, if given, is a zero-filled
    LAUNCH_DTYPE array of the task's length that receives them."""
    n = cfg.launches(task)
    k = cfg.ids(task)
    rec = np.zeros(n, dtype=LAUNCH_DTYPE) if out is None else out
    assert rec.shape == (n,) and rec.dtype == LAUNCH_DTYPE and rec.flags["C_CONTIGUOUS"]
    if n == 0:
        return rec
    tuples = kernel_tuples(cfg, task)
    seq = _id_sequence(cfg, task, n, k)
    # identity fields are the first eight 32-bit words of the record
    words = rec.view("<u4").reshape(n, 16)
    words[:, :8] = tuples[seq]

    rng = _rng(cfg, task, 2)
    # characteristic log-duration and log-gap of each kernel tuple
    z_exec = rng.standard_normal(k)
    z_gap = rng.standard_normal(k)
    e_mu, e_sig = cfg.exec_mu(task), cfg.exec_sigma(task)
    g_mu, g_sig = cfg.gap_mu(task), cfg.gap_sigma(task)
    le = e_mu + e_sig * (cfg.rho_exec * z_exec[seq] + math.sqrt(1 - cfg.rho_exec ** 2) * rng.standard_normal(n))
    exec_ns = np.maximum(1, np.rint(np.exp(le))).astype(np.int64)
    lg = g_mu + g_sig * (cfg.rho_gap * z_gap[seq] + math.sqrt(1 - cfg.rho_gap ** 2) * rng.standard_normal(n))
    gap_ns = np.maximum(0, np.rint(np.exp(lg))).astype(np.int64)
    if cfg.stall_frac > 0:
        u = rng.random(n)
        stall = np.rint(np.exp(cfg.stall_mu + cfg.stall_sigma * rng.standard_normal(n))).astype(np.int64)
        gap_ns = np.where(u < cfg.stall_frac, stall, gap_ns)
    if cfg.zero_gap_frac > 0:
        u = rng.random(n)
        gap_ns = np.where(u < cfg.zero_gap_frac, 0, gap_ns)
    step = exec_ns + gap_ns
    start = np.empty(n, dtype=np.int64)
    start[0] = 0
    np.cumsum(step[:-1], out=start[1:])
    quads = rec.view("<i8").reshape(n, 8)
    quads[:, 4] = start
    np.add(start, exec_ns, out=quads[:, 5])
    if cfg.runs > 1:
        # launch i belongs to run floor(i * runs / n); the time between two runs stays in the timestamps
        words[:, 12] = (np.arange(n, dtype=np.int64) * cfg.runs // n).astype(np.uint32)
    return rec


def task_offsets(cfg: TraceConfig, tasks: Optional[Sequence[int]] = None) -> np.ndarray:
    tasks = range(cfg.n_tasks) if tasks is None else tasks
    off = np.zeros(len(tasks) + 1, dtype=np.uint64)
    np.cumsum([cfg.launches(t) for t in tasks], out=off[1:])
    return off


def build(cfg: TraceConfig, tasks: Optional[Sequence[int]] = None, threads: int = 1,
          out: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Records of the given tasks (default: all) laid out back to back, plus CSR offsets.

    `out`, if given, is a preallocated LAUNCH_DTYPE array of the right length (for example a
    view of pinned host memory) that receives the records."""
    tasks = list(range(cfg.n_tasks) if tasks is None else tasks)
    off = task_offsets(cfg, tasks)
    total = int(off[-1])
    rec = np.zeros(total, dtype=LAUNCH_DTYPE) if out is None else out
    assert rec.shape[0] == total and rec.dtype == LAUNCH_DTYPE

    def fill(i):
        task_records(cfg, tasks[i], out=rec[int(off[i]):int(off[i + 1])])

    if threads <= 1 or len(tasks) <= 1:
        for i in range(len(tasks)):
            fill(i)
    else:
        with ThreadPoolExecutor(threads) as pool:
            list(pool.map(fill, range(len(tasks)), chunksize=max(1, len(tasks) // (threads * 8))))
    return rec, off


def _fill_slot(args):
    """Worker of stream(): regenerates a range of tasks into one slot of the shared staging block."""
    from multiprocessing import shared_memory
    name, index, overrides, lo, hi, slot, slot_records = args
    cfg = config(index, **dict(overrides))
    shm = shared_memory.SharedMemory(name=name)
    try:
        rec = np.ndarray((slot_records,), dtype=LAUNCH_DTYPE, buffer=shm.buf, offset=slot * slot_records * 64)
        at = 0
        for t in range(lo, hi):
            n_t = cfg.launches(t)
            view = rec[at:at + n_t]
            view.view(np.uint8)[:] = 0   # slots are reused
            task_records(cfg, t, out=view)
            at += n_t
        del rec, view
    finally:
        shm.close()
    return slot, lo, hi, at


def stream(cfg: TraceConfig, workers: int = 8, slot_records: int = 1 << 20, slots: Optional[int] = None):
    """Generates a whole workload with worker processes and yields it piecewise:
    (first_record_index, records) for consecutive ranges of whole tasks, in completion order.
    `records` is a view of a reused staging slot: copy it away before asking for the next piece.

    Workers are started with the fork-free "forkserver" method, so the caller may already hold
    a GPU context.  A worker that dies raises here instead of being respawned."""
    import multiprocessing as mp
    from concurrent.futures import FIRST_COMPLETED, ProcessPoolExecutor, wait
    from multiprocessing import shared_memory
    off = task_offsets(cfg)
    lens = (off[1:] - off[:-1]).astype(np.int64)
    if lens.size:
        slot_records = max(slot_records, int(lens.max()))
    slots = slots or 2 * workers
    jobs = []
    lo = 0
    while lo < cfg.n_tasks:
        hi = lo + 1
        while hi < cfg.n_tasks and int(off[hi + 1] - off[lo]) <= slot_records:
            hi += 1
        jobs.append((lo, hi))
        lo = hi
    shm = shared_memory.SharedMemory(create=True, size=max(1, slots * slot_records * 64))
    try:
        ctx = mp.get_context("forkserver")
        with ProcessPoolExecutor(max_workers=workers, mp_context=ctx) as pool:
            free = list(range(slots))
            pending = set()
            nxt = 0
            while nxt < len(jobs) or pending:
                while free and nxt < len(jobs):
                    lo, hi = jobs[nxt]
                    nxt += 1
                    pending.add(pool.submit(_fill_slot, (shm.name, cfg.index, cfg.overrides, lo, hi, free.pop(),
                                                         slot_records)))
                finished, pending = wait(pending, return_when=FIRST_COMPLETED)
                for f in finished:
                    slot, lo, hi, count = f.result()
                    view = np.ndarray((count,), dtype=LAUNCH_DTYPE, buffer=shm.buf, offset=slot * slot_records * 64)
                    yield int(off[lo]), view
                    del view
                    free.append(slot)
    finally:
        shm.close()
        shm.unlink()


def scenarios(cfg: TraceConfig) -> Tuple[np.ndarray, np.ndarray]:
    """(hp_task[S], lp_task[S]) as uint32, task numbers local to the full workload."""
    if cfg.scenario_kind == "pair01":
        return np.array([0], dtype=np.uint32), np.array([1], dtype=np.uint32)
    if cfg.scenario_kind == "grid":
        half = cfg.n_tasks // 2
        hp, lp = np.meshgrid(np.arange(half), np.arange(half, 2 * half), indexing="ij")
        return hp.reshape(-1).astype(np.uint32), lp.reshape(-1).astype(np.uint32)
    if cfg.scenario_kind == "adjacent":
        s = np.arange(cfg.n_tasks // 2, dtype=np.uint32)
        return 2 * s, 2 * s + 1
    return np.zeros(0, dtype=np.uint32), np.zeros(0, dtype=np.uint32)


def prio_scenarios(cfg: TraceConfig, k: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """The scenarios of `scenarios(cfg)` with k low-priority tasks each instead of one: scenario s keeps its own and
    borrows those of the next k-1 scenarios (cyclically).  Priority levels 1..9 follow a fixed pattern in which
    neighbouring entries often share a level.  -> (hp_task[S], lp_offsets[S+1], lp_task[S*k], lp_prio[S*k])."""
    hp, lp = scenarios(cfg)
    n = hp.shape[0]
    if n == 0 or k == 0:
        return hp, np.zeros(n + 1, dtype=np.uint64), np.zeros(0, dtype=np.uint32), np.zeros(0, dtype=np.uint32)
    s = np.arange(n, dtype=np.int64)[:, None]
    j = np.arange(k, dtype=np.int64)[None, :]
    lp_task = lp[(s + j) % n].astype(np.uint32).reshape(-1)
    lp_prio = (1 + ((s // 3 + 2 * (j // 2)) % 9)).astype(np.uint32).reshape(-1)
    lp_offsets = (np.arange(n + 1, dtype=np.uint64) * np.uint64(k)).astype(np.uint64)
    return hp, lp_offsets, lp_task, lp_prio


def gap_offsets(offsets: np.ndarray, hp_task: np.ndarray) -> np.ndarray:
    """Where each scenario's per-gap outputs start: a scenario whose high-priority trace has H
    launches owns max(H - 1, 0) consecutive output slots (one per idle gap between launches)."""
    h = (offsets[1:] - offsets[:-1]).astype(np.int64)[hp_task.astype(np.int64)]
    out = np.zeros(hp_task.shape[0] + 1, dtype=np.uint64)
    np.cumsum(np.maximum(h - 1, 0), out=out[1:])
    return out
