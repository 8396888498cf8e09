"""Traces that hold several measured runs of a task (Section 3.2: statistics over all T runs, N - 1 idle times per
run): fikit_profile and fikit_measure against the oracle, every field, on all the paths a task can take."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2311_10359_amd import binding, traces
from parity_util import DEV, check_gapfill, check_profile
from test_oracle_pins import make_records

pytestmark = pytest.mark.gpu


def cases():
    return {
        "cfg0_tiny_3_runs": traces.config(0, runs=3),
        "cfg1_medium_4x20000_4_runs": traces.config(1, n_tasks=4, launches=20000, runs=4),    # long tasks: tile partition + units
        "cfg1_medium_2x8193_2_runs": traces.config(1, n_tasks=2, launches=8193, runs=2),
        "cfg2_skewed_2x100000_7_runs": traces.config(2, n_tasks=2, launches=100000, runs=7),  # general path
        "cfg3_large_3x30000_10_runs": traces.config(3, n_tasks=3, launches=30000, runs=10),
        "cfg4_batched_64_5_runs": traces.config(4, n_tasks=64, runs=5),                       # the shapes the benchmark runs in
        "cfg4_batched_small_1000_runs": traces.config(4, n_tasks=40, hp_launches=500, lp_launches=1500, runs=400),
    }


@pytest.mark.parametrize("name", list(cases()))
def test_profile_with_runs_matches_oracle(name):
    cfg = cases()[name]
    print(f"case {name}: {cfg.n_records} records, {cfg.n_tasks} tasks, {cfg.runs} runs each", flush=True)
    rec, off = traces.build(cfg, threads=4)
    prof, d_off, o_prof = check_profile(rec, off)
    n_runs = sum(len(np.unique(rec["run"][int(off[t]):int(off[t + 1])])) for t in range(cfg.n_tasks))
    rows = binding.rows_to_numpy(prof.rows)
    assert int(rows["gap"]["count"].sum()) == rec.shape[0] - n_runs
    # per-launch measurements: no idle time after the last launch of a run
    d_exec, d_gap = binding.fikit_measure(binding.to_device_records(rec, DEV), d_off)
    ex, gp = oracle.measure(rec, off)
    assert np.array_equal(d_exec.cpu().numpy(), ex) and np.array_equal(d_gap.cpu().numpy(), gp)
    assert int((gp < 0).sum()) == n_runs
    # the gap fill reads the rows only: same comparison as for one-run traces
    hp, lp = traces.scenarios(cfg)
    if hp.size:
        check_gapfill(prof, d_off, off, o_prof, hp, lp, cfg.margin_ns, cfg.min_gap_ns)


def test_runs_hand_worked(golden_dir):
    with open(os.path.join(golden_dir, "p1_hand_worked.json")) as f:
        g1 = json.load(f)
    with open(os.path.join(golden_dir, "p10_runs_hand_worked.json")) as f:
        g = json.load(f)
    k = g1["kernels"]
    hp = make_records([(k[n]["name_id"], k[n]["grid"], k[n]["block"], k[n]["shmem"], s, e) for n, s, e in g1["hp_trace"]])
    for case in g["cases"].values():
        rec = hp.copy()
        rec["run"] = case["run_of_launch"]
        prof, _, _ = check_profile(rec, np.array([0, 12], dtype=np.uint64))
        rows = binding.rows_to_numpy(prof.rows)
        for r, name in zip(rows, g1["rows_in_order"][:3]):
            assert [int(r["gap"][f]) for f in g["_stats_order"]] == case["gap"][name]
            assert [int(r["exec"][f]) for f in g["_stats_order"]] == g1["rows"][name]["exec"]


def test_replay_refuses_a_high_priority_trace_with_several_runs():
    cfg = traces.config(4, n_tasks=8, hp_launches=200, lp_launches=600, runs=2)
    rec, off = traces.build(cfg)
    d_off = binding.to_device_u64(off, DEV)
    d_rec = binding.to_device_records(rec, DEV)
    prof = binding.fikit_profile(d_rec, d_off)
    _, d_gap = binding.fikit_measure(d_rec, d_off)
    hp, lp = traces.scenarios(cfg)
    go = traces.gap_offsets(off, hp)
    with pytest.raises(binding.FikitError) as e:
        binding.fikit_gapfill_replay(prof.ids, d_off, prof.rows, prof.task_row_offsets, d_gap, binding.to_device_u32(hp, DEV),
                                     binding.to_device_u32(lp, DEV), binding.to_device_u64(go, DEV), margin_ns=500, min_gap_ns=0,
                                     feedback=True)
    assert e.value.status == binding.FIKIT_INVALID_ARG
