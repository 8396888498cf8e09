"""Per-launch measurement and the replay of the gap fill against actual idle times: HIP library vs CPU
oracle, element by element, through the C ABI (needs an MI355X)."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2311_10359_amd import binding, traces
from parity_util import DEV, check_profile
from test_gpu_parity import all_pairs, mixed_trace, ragged_trace
from test_oracle_pins import replay_inputs

pytestmark = pytest.mark.gpu


def check_measure(rec, off):
    ex, gp = oracle.measure(rec, off)
    d_ex, d_gp = binding.fikit_measure(binding.to_device_records(rec, DEV), binding.to_device_u64(off, DEV))
    torch.cuda.synchronize()
    assert np.array_equal(d_ex.cpu().numpy(), ex), "execution times differ"
    assert np.array_equal(d_gp.cpu().numpy(), gp), "idle times differ"
    return d_gp, gp


def check_replay(prof, d_off, off, o_prof, d_gap, gap, hp, lp, margin, min_gap, out=None, predictor=0):
    o_ids, o_rows, o_tro = o_prof
    go = traces.gap_offsets(off, hp)
    d_hp, d_lp, d_go = binding.to_device_u32(hp, DEV), binding.to_device_u32(lp, DEV), binding.to_device_u64(go, DEV)
    for feedback in (False, True):
        exp = oracle.replay(o_ids, off, o_rows, o_tro, gap, hp, lp, margin, min_gap, feedback, go, predictor=predictor)
        got = binding.fikit_gapfill_replay(prof.ids, d_off, prof.rows, prof.task_row_offsets, d_gap, d_hp, d_lp, d_go,
                                           margin_ns=margin, min_gap_ns=min_gap, feedback=feedback,
                                           predictor=predictor, n_gaps=int(go[-1]), out=out)
        torch.cuda.synchronize()
        fc, fn = binding.u32_to_numpy(got.fill_count), got.filled_ns.cpu().numpy()
        bad = np.nonzero(fc != exp[0])[0]
        assert bad.size == 0, f"feedback={feedback}: fill_count differs at {bad[:5]}: {fc[bad[:5]]} vs {exp[0][bad[:5]]}"
        bad = np.nonzero(fn != exp[1])[0]
        assert bad.size == 0, f"feedback={feedback}: filled_ns differs at {bad[:5]}"
        delay = got.hp_delay_ns.cpu().numpy()
        bad = np.nonzero(delay != exp[2])[0]
        assert bad.size == 0, f"feedback={feedback}: hp_delay_ns differs at {bad[:5]}: {delay[bad[:5]]} vs {exp[2][bad[:5]]}"
        assert np.array_equal(binding.u64_to_numpy(got.lp_placed), exp[3]), f"feedback={feedback}: lp_placed differs"


def test_measure_matches_oracle():
    for cfg in (traces.config(0), traces.config(1, n_tasks=3, launches=5000), traces.config(4, n_tasks=6, hp_launches=300, lp_launches=700)):
        rec, off = traces.build(cfg, threads=2)
        check_measure(rec, off)
    rec, off = ragged_trace(7, [0, 1, 0, 2, 255, 256, 257, 0, 1000, 1, 0], 5)
    check_measure(rec, off)
    # empty input, and a record that ends before it starts
    ex, gp = binding.fikit_measure(torch.empty((0, 64), dtype=torch.uint8, device=DEV), binding.to_device_u64(np.zeros(1, np.uint64), DEV))
    assert ex.numel() == 0 and gp.numel() == 0
    rec["end_ns"][5] = rec["start_ns"][5] - 1
    with pytest.raises(binding.FikitError) as e:
        binding.fikit_measure(binding.to_device_records(rec, DEV), binding.to_device_u64(off, DEV))
    assert e.value.status == binding.FIKIT_BAD_RECORD


def test_replay_hand_worked(golden_dir):
    with open(os.path.join(golden_dir, "p6_replay_hand_worked.json")) as f:
        golden = json.load(f)
    ids, off, rows, tro = replay_inputs(golden)
    hp, lp = np.array([0], dtype=np.uint32), np.array([1], dtype=np.uint32)
    go = traces.gap_offsets(off, hp)
    d = dict(ids=binding.to_device_u64(ids, DEV), off=binding.to_device_u64(off, DEV),
             rows=torch.from_numpy(rows.view(np.uint8).reshape(-1, 128)).to(DEV), tro=binding.to_device_u64(tro, DEV),
             hp=binding.to_device_u32(hp, DEV), lp=binding.to_device_u32(lp, DEV), go=binding.to_device_u64(go, DEV))
    for case in golden["cases"]:
        actual = np.array(case["actual_gap_ns"] + [-1] + [1] * (len(golden["lp_ids"]) - 1) + [-1], dtype=np.int64)
        for feedback, key in ((False, "no_feedback"), (True, "feedback")):
            got = binding.fikit_gapfill_replay(d["ids"], d["off"], d["rows"], d["tro"], torch.from_numpy(actual).to(DEV),
                                               d["hp"], d["lp"], d["go"], margin_ns=case["margin_ns"],
                                               min_gap_ns=case["min_gap_ns"], feedback=feedback)
            exp = case[key]
            assert binding.u32_to_numpy(got.fill_count).tolist() == exp["fill_count"], (case, key)
            assert got.filled_ns.cpu().tolist() == exp["filled_ns"], (case, key)
            assert int(got.hp_delay_ns[0]) == exp["hp_delay_ns"] and int(got.lp_placed[0]) == exp["lp_placed"], (case, key)


@pytest.mark.parametrize("name", ["cfg0_tiny", "cfg1_medium_3x20000", "cfg4_batched_small"])
def test_replay_small_configs(name):
    cfg = {"cfg0_tiny": traces.config(0), "cfg1_medium_3x20000": traces.config(1, n_tasks=4, launches=20000),
           "cfg4_batched_small": traces.config(4, n_tasks=40, hp_launches=500, lp_launches=1500)}[name]
    rec, off = traces.build(cfg, threads=4)
    prof, d_off, o_prof = check_profile(rec, off)
    d_gap, gap = check_measure(rec, off)
    hp, lp = traces.scenarios(cfg)
    for margin, min_gap in ((cfg.margin_ns, cfg.min_gap_ns), (0, 100000)):
        check_replay(prof, d_off, off, o_prof, d_gap, gap, hp, lp, margin, min_gap)


def test_replay_many_scenarios():
    cfg = traces.config(4, n_tasks=72, hp_launches=301, lp_launches=1203)
    rec, off = traces.build(cfg, threads=4)
    prof, d_off, o_prof = check_profile(rec, off)
    d_gap, gap = check_measure(rec, off)
    hp, lp = all_pairs(range(cfg.n_tasks))
    for margin, min_gap in ((cfg.margin_ns, cfg.min_gap_ns), (0, 100000), (40000, 0)):
        print(f"{hp.size} scenarios, margin {margin}, min gap {min_gap}", flush=True)
        check_replay(prof, d_off, off, o_prof, d_gap, gap, hp, lp, margin, min_gap)
    check_replay(prof, d_off, off, o_prof, d_gap, gap, hp, lp, cfg.margin_ns, cfg.min_gap_ns, predictor=binding.FIKIT_PREDICT_MEAN)


def test_replay_ragged_tasks_and_unaligned_outputs():
    lens = [0, 1, 2, 3, 7, 8, 9, 15, 16, 17, 31, 33, 63, 64, 65, 100, 127, 129, 255, 257, 500, 1000, 1001, 2047,
            0, 5, 6, 40, 41, 42, 43, 44] + [11 * k + 1 for k in range(32)]
    rec, off = ragged_trace(4242, lens, 9)
    prof, d_off, o_prof = check_profile(rec, off)
    d_gap, gap = check_measure(rec, off)
    hp, lp = all_pairs(range(len(lens)))
    check_replay(prof, d_off, off, o_prof, d_gap, gap, hp, lp, 300, 0)
    check_replay(prof, d_off, off, o_prof, d_gap, gap, hp, lp, 0, 5000)
    n_gaps = int(traces.gap_offsets(off, hp)[-1])
    out = binding.Replay(torch.empty(n_gaps + 1, dtype=torch.int32, device=DEV)[1:],
                         torch.empty(n_gaps + 1, dtype=torch.int64, device=DEV)[1:],
                         torch.empty(hp.size, dtype=torch.int64, device=DEV), torch.empty(hp.size, dtype=torch.int64, device=DEV))
    check_replay(prof, d_off, off, o_prof, d_gap, gap, hp, lp, 300, 0, out=out)


def test_replay_mixed_task_shapes():
    rec, off, lens = mixed_trace(22, 64, max_len=4097, wide=False)
    prof, d_off, o_prof = check_profile(rec, off)
    d_gap, gap = check_measure(rec, off)
    hp, lp = all_pairs(range(len(lens)))
    check_replay(prof, d_off, off, o_prof, d_gap, gap, hp, lp, 100, 0)
    check_replay(prof, d_off, off, o_prof, d_gap, gap, hp, lp, 0, 2000, predictor=binding.FIKIT_PREDICT_MEAN)


def test_replay_error_statuses():
    lens = [40 + k for k in range(8)]
    rec, off = ragged_trace(5, lens, 4)
    prof, d_off, o_prof = check_profile(rec, off)
    d_gap, gap = check_measure(rec, off)
    hp, lp = all_pairs(range(len(lens)))
    go = traces.gap_offsets(off, hp)
    args = (prof.ids, d_off, prof.rows, prof.task_row_offsets)
    tail = (binding.to_device_u32(hp, DEV), binding.to_device_u32(lp, DEV), binding.to_device_u64(go, DEV))
    # a negative actual idle time where a gap is
    bad = gap.copy()
    bad[3] = -5
    with pytest.raises(binding.FikitError) as e:
        binding.fikit_gapfill_replay(*args, torch.from_numpy(bad).to(DEV), *tail, margin_ns=0, min_gap_ns=0, feedback=True)
    assert e.value.status == binding.FIKIT_INVALID_ARG
    with pytest.raises(oracle.OracleError) as oe:
        oracle.replay(*o_prof[:1], off, o_prof[1], o_prof[2], bad, hp, lp, 0, 0, True, go)
    assert oe.value.status == oracle.INVALID_ARG


def test_replay_predictions_beyond_32_bits():
    """A prediction of 2^32 - 1 ns or more: the 64-bit kernels take the call; results are the oracle's."""
    lens = [40 + k for k in range(8)]
    rec, off = ragged_trace(5, lens, 4)
    slow = rec["name_id"] == 1
    ex = (rec["end_ns"] - rec["start_ns"]).astype(np.int64)
    ex[slow] += 5_000_000_000
    idle = np.where(rec["name_id"] == 2, 11_000_000_000, 1000)             # a kernel whose idle time such kernels fit into
    start = np.cumsum(ex + idle) - (ex + idle)
    rec["start_ns"], rec["end_ns"] = start, start + ex
    prof, d_off, o_prof = check_profile(rec, off)
    d_gap, gap = check_measure(rec, off)
    hp, lp = all_pairs(range(len(lens)))
    for margin, min_gap in ((0, 0), (500, 2000), (10**10, 0)):
        check_replay(prof, d_off, off, o_prof, d_gap, gap, hp, lp, margin, min_gap)
    # actual idle times that differ from the predictions (shorter and longer), and a negative one
    rng = np.random.default_rng(9)
    other = np.where(gap >= 0, (gap * rng.uniform(0.2, 1.8, gap.size)).astype(np.int64), gap)
    check_replay(prof, d_off, off, o_prof, torch.from_numpy(other).to(DEV), other, hp, lp, 0, 0)
    bad = gap.copy()
    bad[3] = -5
    go = traces.gap_offsets(off, hp)
    with pytest.raises(binding.FikitError) as e:
        binding.fikit_gapfill_replay(prof.ids, d_off, prof.rows, prof.task_row_offsets, torch.from_numpy(bad).to(DEV),
                                     binding.to_device_u32(hp, DEV), binding.to_device_u32(lp, DEV), binding.to_device_u64(go, DEV),
                                     margin_ns=0, min_gap_ns=0, feedback=False)
    assert e.value.status == binding.FIKIT_INVALID_ARG
