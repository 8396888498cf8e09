"""Profiles merged over runs: HIP library vs CPU oracle, byte for byte, through the C ABI (needs an MI355X)."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2311_10359_amd import binding, traces
from parity_util import DEV, check_gapfill, run_profile_gpu
from test_oracle_pins import offsets_of, rows_from_json, split_runs

pytestmark = pytest.mark.gpu


def to_dev_rows(rows):
    return torch.from_numpy(np.ascontiguousarray(rows).view(np.uint8).reshape(-1, 128)).to(DEV)


def check_merge(a, ao, b, bo):
    exp, exp_off = oracle.profile_merge(a, ao, b, bo)
    got = binding.fikit_profile_merge(to_dev_rows(a), binding.to_device_u64(ao, DEV), to_dev_rows(b), binding.to_device_u64(bo, DEV))
    torch.cuda.synchronize()
    assert got.n_rows == exp.shape[0]
    assert np.array_equal(binding.u64_to_numpy(got.task_row_offsets), exp_off)
    rows = binding.rows_to_numpy(got.rows)
    if rows.tobytes() != exp.tobytes():
        for f in ("kernel_id", "task"):
            bad = np.nonzero(rows[f] != exp[f])[0]
            assert bad.size == 0, f"{f} differs at {bad[:5]}"
        for blk in ("exec", "gap"):
            for f in ("count", "sum", "min", "max", "p50", "p95"):
                bad = np.nonzero(rows[blk][f] != exp[blk][f])[0]
                assert bad.size == 0, f"{blk}.{f} differs at {bad[:5]}: {rows[blk][f][bad[:5]]} vs {exp[blk][f][bad[:5]]}"
        raise AssertionError("rows differ in reserved bytes")
    return got


def test_merge_hand_worked(golden_dir):
    with open(os.path.join(golden_dir, "p9_merge_hand_worked.json")) as f:
        golden = json.load(f)
    n_tasks = golden["n_tasks"]
    a, b, exp = rows_from_json(golden["a"]), rows_from_json(golden["b"]), rows_from_json(golden["merged"])
    got = binding.fikit_profile_merge(to_dev_rows(a), binding.to_device_u64(offsets_of(a, n_tasks), DEV), to_dev_rows(b),
                                      binding.to_device_u64(offsets_of(b, n_tasks), DEV))
    assert binding.rows_to_numpy(got.rows).tobytes() == exp.tobytes()
    assert np.array_equal(binding.u64_to_numpy(got.task_row_offsets), offsets_of(exp, n_tasks))


def random_rows(rng, n_tasks, max_ids, id_pool):
    """A row table with random (plausible) statistics; the IDs of a task are a random subset of the task's pool."""
    rows, off = [], [0]
    for t in range(n_tasks):
        k = int(rng.integers(0, max_ids + 1))
        ids = np.sort(rng.choice(id_pool[t], size=min(k, id_pool[t].size), replace=False))
        r = np.zeros(ids.size, dtype=oracle.ROW_DTYPE)
        r["kernel_id"], r["task"] = ids, t
        for blk in ("exec", "gap"):
            cnt = rng.integers(0 if blk == "gap" else 1, 50, ids.size)
            lo = rng.integers(0, 1000, ids.size)
            hi = lo + rng.integers(0, 10**6, ids.size)
            p50 = lo + (hi - lo) // 3
            has = cnt > 0
            r[blk]["count"] = cnt
            r[blk]["sum"] = np.where(has, rng.integers(0, 2**62, ids.size), 0)
            for f, v in (("min", lo), ("max", hi), ("p50", p50), ("p95", hi)):
                r[blk][f] = np.where(has, v, 0)
        rows.append(r)
        off.append(off[-1] + ids.size)
    return np.concatenate(rows) if rows else np.zeros(0, oracle.ROW_DTYPE), np.array(off, dtype=np.uint64)


@pytest.mark.parametrize("n_tasks,max_ids,pool", [(1, 5, 8), (40, 300, 400), (7, 5000, 6000), (300, 40, 45), (3, 9000, 9100)])
def test_merge_random_tables(n_tasks, max_ids, pool):
    rng = np.random.default_rng(n_tasks * 1000 + max_ids)
    id_pool = [np.unique(rng.integers(0, 2**64, pool, dtype=np.uint64)) for _ in range(n_tasks)]
    a, ao = random_rows(rng, n_tasks, max_ids, id_pool)
    b, bo = random_rows(rng, n_tasks, max_ids, id_pool)
    print(f"{n_tasks} tasks, {a.shape[0]} + {b.shape[0]} rows", flush=True)
    check_merge(a, ao, b, bo)
    empty, zero = np.zeros(0, dtype=oracle.ROW_DTYPE), np.zeros(n_tasks + 1, dtype=np.uint64)
    check_merge(a, ao, empty, zero)
    check_merge(empty, zero, b, bo)
    check_merge(a, ao, a, ao)


def test_merge_of_runs_feeds_the_gap_fill():
    cfg = traces.config(4, n_tasks=40, hp_launches=500, lp_launches=1500)
    rec, off = traces.build(cfg, threads=4)
    (r1, o1), (r2, o2) = split_runs(rec, off, 0.5)
    p1, _ = run_profile_gpu(r1, o1)
    p2, _ = run_profile_gpu(r2, o2)
    merged = binding.fikit_profile_merge(p1.rows, p1.task_row_offsets, p2.rows, p2.task_row_offsets)
    torch.cuda.synchronize()
    _, rows1, tro1 = oracle.profile(r1, o1)
    _, rows2, tro2 = oracle.profile(r2, o2)
    o_rows, o_tro = oracle.profile_merge(rows1, tro1, rows2, tro2)
    assert binding.rows_to_numpy(merged.rows).tobytes() == o_rows.tobytes()
    # the merged table drives the gap fill of the whole traces, with the means as predictions
    whole, d_off = run_profile_gpu(rec, off)
    o_ids, _, _ = oracle.profile(rec, off)
    hp, lp = traces.scenarios(cfg)
    prof = whole._replace(rows=merged.rows, task_row_offsets=merged.task_row_offsets, n_rows=merged.n_rows)
    check_gapfill(prof, d_off, off, (o_ids, o_rows, o_tro), hp, lp, cfg.margin_ns, cfg.min_gap_ns,
                  predictor=binding.FIKIT_PREDICT_MEAN)


def test_merge_argument_errors():
    rng = np.random.default_rng(1)
    id_pool = [np.unique(rng.integers(0, 2**64, 50, dtype=np.uint64)) for _ in range(4)]
    a, ao = random_rows(rng, 4, 30, id_pool)
    b, bo = random_rows(rng, 4, 30, id_pool)
    exp, _ = oracle.profile_merge(a, ao, b, bo)

    def call(a_, ao_, b_, bo_, **kw):
        return binding.fikit_profile_merge(to_dev_rows(a_), binding.to_device_u64(ao_, DEV), to_dev_rows(b_),
                                           binding.to_device_u64(bo_, DEV), **kw)

    with pytest.raises(binding.FikitError) as e:
        call(a, ao, b, bo, row_capacity=exp.shape[0] - 1)
    assert e.value.status == binding.FIKIT_ROW_CAPACITY and e.value.n_rows == exp.shape[0]
    t_with_two = int(np.nonzero(np.diff(ao.astype(np.int64)) >= 2)[0][0])
    first = int(ao[t_with_two])
    wrong_task = a.copy()
    wrong_task["task"][first] = (t_with_two + 1) % 4
    unsorted = a.copy()
    unsorted["kernel_id"][first], unsorted["kernel_id"][first + 1] = a["kernel_id"][first + 1], a["kernel_id"][first]
    twice = a.copy()
    twice["kernel_id"][first + 1] = a["kernel_id"][first]
    bad_off = ao.copy()
    bad_off[1], bad_off[2] = ao[2], ao[1]
    for bad_a, bad_ao in ((wrong_task, ao), (unsorted, ao), (twice, ao), (a, bad_off) if ao[1] != ao[2] else (wrong_task, ao)):
        with pytest.raises(binding.FikitError) as e:
            call(bad_a, bad_ao, b, bo)
        assert e.value.status == binding.FIKIT_INVALID_ARG
        with pytest.raises(binding.FikitError) as e:
            call(b, bo, bad_a, bad_ao)
        assert e.value.status == binding.FIKIT_INVALID_ARG
    call(a, ao, b, bo)
