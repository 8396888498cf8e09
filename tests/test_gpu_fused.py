"""fikit_profile_gapfill (the two calls of the hot path as one) against the oracle: every output of the profile and of
the gap fill, bit for bit, where the profile's own kernels write the predictions (many scenarios, tasks that one
workgroup holds) and where they do not (few scenarios, long tasks, tasks left to the sort, predictions beyond 32 bits)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_10359_amd import binding, traces
from parity_util import DEV, assert_profile_equal
from test_gpu_parity import all_pairs, mixed_trace, ragged_trace

pytestmark = pytest.mark.gpu


def check_fused(rec, off, hp, lp, margin, min_gap, predictor=0, o_prof=None):
    o_ids, o_rows, o_tro = o_prof if o_prof is not None else oracle.profile(rec, off)
    go = traces.gap_offsets(off, hp)
    exp = oracle.gapfill(o_ids, off, o_rows, o_tro, hp, lp, margin, min_gap, go, predictor=predictor)
    prof, got = binding.fikit_profile_gapfill(binding.to_device_records(rec, DEV), binding.to_device_u64(off, DEV),
                                              binding.to_device_u32(hp, DEV), binding.to_device_u32(lp, DEV),
                                              binding.to_device_u64(go, DEV), margin_ns=margin, min_gap_ns=min_gap,
                                              predictor=predictor)
    torch.cuda.synchronize()
    assert_profile_equal(prof, o_ids, o_rows, o_tro)
    fc = binding.u32_to_numpy(got.fill_count)
    bad = np.nonzero(fc != exp[0])[0]
    assert bad.size == 0, f"fill_count differs at {bad[:5]}: {fc[bad[:5]]} vs {exp[0][bad[:5]]}"
    assert np.array_equal(got.filled_ns.cpu().numpy(), exp[1]), "filled_ns differs"
    assert np.array_equal(got.lp_completion_ns.cpu().numpy(), exp[2]), "lp_completion_ns differs"
    assert np.array_equal(binding.u64_to_numpy(got.lp_placed), exp[3]), "lp_placed differs"
    return (o_ids, o_rows, o_tro)


def test_batched_workload_shape():
    """The benchmark's shape at a reduced size: a high-priority trace and a low-priority queue per scenario, one lane
    per scenario; launches beyond 4096 and 8192 so that all three shapes of the task kernel write predictions."""
    for hp_l, lp_l in ((300, 1200), (4100, 8300)):
        cfg = traces.config(4, n_tasks=8400 if hp_l == 300 else 8200, hp_launches=hp_l, lp_launches=lp_l)
        rec, off = traces.build(cfg, threads=4)
        hp, lp = traces.scenarios(cfg)
        assert hp.size >= 4096
        o = check_fused(rec, off, hp, lp, cfg.margin_ns, cfg.min_gap_ns)
        check_fused(rec, off, hp, lp, 0, 100000, predictor=binding.FIKIT_PREDICT_MEAN, o_prof=o)


def test_shared_tasks_in_both_roles():
    """Every ordered pair of 72 tasks (a task against itself included): tasks are trace and queue at once."""
    cfg = traces.config(4, n_tasks=72, hp_launches=301, lp_launches=1203)
    rec, off = traces.build(cfg, threads=4)
    hp, lp = all_pairs(range(cfg.n_tasks))
    o = check_fused(rec, off, hp, lp, cfg.margin_ns, cfg.min_gap_ns)
    check_fused(rec, off, hp, lp, 40000, 0, predictor=binding.FIKIT_PREDICT_MEAN, o_prof=o)


def test_mixed_task_shapes():
    """Every size class side by side, tasks with too many IDs for a workgroup, heavy ties: some tasks' predictions
    come from the profile's kernels, the others' from the gap fill's."""
    rec, off, lens = mixed_trace(21, 64, max_len=20000, wide=False)
    hp, lp = all_pairs(range(len(lens)))
    o = check_fused(rec, off, hp, lp, 100, 0)
    check_fused(rec, off, hp, lp, 0, 2000, predictor=binding.FIKIT_PREDICT_MEAN, o_prof=o)


def test_ragged_and_empty_tasks():
    lens = [0, 1, 2, 3, 7, 8, 9, 15, 16, 17, 31, 33, 63, 64, 65, 100, 127, 129, 255, 257, 500, 1000, 1001, 2047,
            0, 5, 6, 40, 41, 42, 43, 44] + [11 * k + 1 for k in range(32)]
    rec, off = ragged_trace(4242, lens, 9)
    hp, lp = all_pairs(range(len(lens)))
    check_fused(rec, off, hp, lp, 300, 0)


def test_few_scenarios_and_none():
    """Fewer scenarios than the one-lane kernels are used for: the call is the two calls; no scenario: the profile."""
    cfg = traces.config(1, n_tasks=8, launches=3000)
    rec, off = traces.build(cfg, threads=4)
    hp, lp = traces.scenarios(cfg)
    check_fused(rec, off, hp, lp, cfg.margin_ns, cfg.min_gap_ns)
    none = np.zeros(0, dtype=np.uint32)
    check_fused(rec, off, none, none, 0, 0)


def test_predictions_beyond_32_bits():
    lens = [40 + k for k in range(64)]
    rec, off = ragged_trace(99, lens, 4)
    ex = (rec["end_ns"] - rec["start_ns"]).astype(np.int64)
    ex[rec["name_id"] == 1] += 5_000_000_000
    gp = np.full(rec.shape[0], 1000, dtype=np.int64)
    gp[rec["name_id"] == 2] = 6_000_000_000
    start = np.cumsum(ex + gp) - (ex + gp)
    rec["start_ns"] = start
    rec["end_ns"] = start + ex
    hp, lp = all_pairs(range(len(lens)))
    check_fused(rec, off, hp, lp, 300, 0)


def test_runs_and_errors():
    """A trace with run numbers (no idle time across runs) through the fused call; a bad record is reported."""
    cfg = traces.config(4, n_tasks=8400, hp_launches=64, lp_launches=96, runs=3)
    rec, off = traces.build(cfg, threads=4)
    hp, lp = traces.scenarios(cfg)
    check_fused(rec, off, hp, lp, cfg.margin_ns, cfg.min_gap_ns)
    bad = rec.copy()
    bad["end_ns"][5] = bad["start_ns"][5] - 1
    go = traces.gap_offsets(off, hp)
    with pytest.raises(binding.FikitError) as e:
        binding.fikit_profile_gapfill(binding.to_device_records(bad, DEV), binding.to_device_u64(off, DEV),
                                      binding.to_device_u32(hp, DEV), binding.to_device_u32(lp, DEV),
                                      binding.to_device_u64(go, DEV), margin_ns=0, min_gap_ns=0)
    assert e.value.status == -4
