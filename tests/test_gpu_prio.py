"""Gap filling with several low-priority tasks in priority queues (BestPrioFit): HIP library vs CPU oracle,
element by element, through the C ABI (needs an MI355X)."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2311_10359_amd import binding, traces
from parity_util import DEV, check_profile
from test_gpu_parity import mixed_trace, ragged_trace
from test_oracle_pins import prio_inputs

pytestmark = pytest.mark.gpu


def prio_lists(rng, n_tasks, n_scen, k_max, same_level=0.5):
    """Scenarios with 0..k_max low-priority tasks each, many of them on one level."""
    hp = rng.integers(0, n_tasks, n_scen).astype(np.uint32)
    k = rng.integers(0, k_max + 1, n_scen)
    lo = np.zeros(n_scen + 1, dtype=np.uint64)
    np.cumsum(k, out=lo[1:])
    lt = rng.integers(0, n_tasks, int(lo[-1])).astype(np.uint32)
    lq = rng.integers(1, 10, int(lo[-1])).astype(np.uint32)
    lq[rng.random(lq.shape[0]) < same_level] = 4
    return hp, lo, lt, lq


def check_prio(prof, d_off, off, o_prof, hp, lo, lt, lq, margin, min_gap, predictor=0, out=None):
    o_ids, o_rows, o_tro = o_prof
    go = traces.gap_offsets(off, hp)
    exp = oracle.prio_fill(o_ids, off, o_rows, o_tro, hp, lo, lt, lq, margin, min_gap, go, predictor=predictor)
    got = binding.fikit_prio_fill(prof.ids, d_off, prof.rows, prof.task_row_offsets, binding.to_device_u32(hp, DEV),
                                  binding.to_device_u64(lo, DEV), binding.to_device_u32(lt, DEV), binding.to_device_u32(lq, DEV),
                                  binding.to_device_u64(go, DEV), margin_ns=margin, min_gap_ns=min_gap, predictor=predictor,
                                  n_gaps=int(go[-1]), out=out)
    torch.cuda.synchronize()
    fc, fn = binding.u32_to_numpy(got.fill_count), got.filled_ns.cpu().numpy()
    bad = np.nonzero(fc != exp[0])[0]
    assert bad.size == 0, f"fill_count differs at {bad[:5]}: {fc[bad[:5]]} vs {exp[0][bad[:5]]}"
    bad = np.nonzero(fn != exp[1])[0]
    assert bad.size == 0, f"filled_ns differs at {bad[:5]}: {fn[bad[:5]]} vs {exp[1][bad[:5]]}"
    placed, placed_ns = binding.u64_to_numpy(got.lp_placed), got.lp_placed_ns.cpu().numpy()
    bad = np.nonzero(placed != exp[2])[0]
    assert bad.size == 0, f"lp_placed differs at {bad[:5]}: {placed[bad[:5]]} vs {exp[2][bad[:5]]}"
    bad = np.nonzero(placed_ns != exp[3])[0]
    assert bad.size == 0, f"lp_placed_ns differs at {bad[:5]}"
    return got, exp


@pytest.mark.parametrize("case", ["abc", "equal_priority", "longest_fit"])
def test_prio_hand_worked(golden_dir, case):
    with open(os.path.join(golden_dir, "p7_prio_fill_hand_worked.json")) as f:
        golden = json.load(f)
    exp = golden["cases"][case]
    ids, off, rows, tro, hp, lo, lt, lq = prio_inputs(golden["hp_launches"], golden["hp_gap"], exp["lp"])
    go = traces.gap_offsets(off, hp)
    got = binding.fikit_prio_fill(binding.to_device_u64(ids, DEV), binding.to_device_u64(off, DEV),
                                  torch.from_numpy(rows.view(np.uint8).reshape(-1, 128)).to(DEV), binding.to_device_u64(tro, DEV),
                                  binding.to_device_u32(hp, DEV), binding.to_device_u64(lo, DEV), binding.to_device_u32(lt, DEV),
                                  binding.to_device_u32(lq, DEV), binding.to_device_u64(go, DEV), margin_ns=0, min_gap_ns=0)
    assert binding.u32_to_numpy(got.fill_count).tolist() == exp["fill_count"]
    assert got.filled_ns.cpu().tolist() == exp["filled_ns"]
    assert got.lp_placed.cpu().tolist() == exp["lp_placed"] and got.lp_placed_ns.cpu().tolist() == exp["lp_placed_ns"]


@pytest.mark.parametrize("name", ["cfg0_tiny", "cfg1_medium_4x20000", "cfg4_batched_small"])
def test_prio_small_configs(name):
    cfg = {"cfg0_tiny": traces.config(0), "cfg1_medium_4x20000": traces.config(1, n_tasks=4, launches=20000),
           "cfg4_batched_small": traces.config(4, n_tasks=40, hp_launches=500, lp_launches=1500)}[name]
    rec, off = traces.build(cfg, threads=4)
    prof, d_off, o_prof = check_profile(rec, off)
    rng = np.random.default_rng(11)
    for k_max, n_scen in ((1, 70), (2, 300), (3, 300), (4, 257), (7, 130), (13, 70), (30, 40), (64, 9)):
        hp, lo, lt, lq = prio_lists(rng, cfg.n_tasks, n_scen, k_max)
        print(f"{name}: up to {k_max} low-priority tasks, {n_scen} scenarios, {lt.size} entries", flush=True)
        check_prio(prof, d_off, off, o_prof, hp, lo, lt, lq, cfg.margin_ns, cfg.min_gap_ns)
    hp, lo, lt, lq = prio_lists(rng, cfg.n_tasks, 200, 4)
    check_prio(prof, d_off, off, o_prof, hp, lo, lt, lq, 0, 100000)
    check_prio(prof, d_off, off, o_prof, hp, lo, lt, lq, 40000, 0, predictor=binding.FIKIT_PREDICT_MEAN)


def test_prio_one_task_is_the_gap_fill():
    cfg = traces.config(4, n_tasks=72, hp_launches=301, lp_launches=1203)
    rec, off = traces.build(cfg, threads=4)
    prof, d_off, o_prof = check_profile(rec, off)
    hp, lp = traces.scenarios(cfg)
    lo = np.arange(hp.size + 1, dtype=np.uint64)
    lq = np.random.default_rng(3).integers(1, 10, hp.size).astype(np.uint32)
    got, _ = check_prio(prof, d_off, off, o_prof, hp, lo, lp, lq, cfg.margin_ns, cfg.min_gap_ns)
    go = traces.gap_offsets(off, hp)
    ref = binding.fikit_gapfill(prof.ids, d_off, prof.rows, prof.task_row_offsets, binding.to_device_u32(hp, DEV),
                                binding.to_device_u32(lp, DEV), binding.to_device_u64(go, DEV), margin_ns=cfg.margin_ns,
                                min_gap_ns=cfg.min_gap_ns)
    assert torch.equal(got.fill_count, ref.fill_count) and torch.equal(got.filled_ns, ref.filled_ns)
    assert torch.equal(got.lp_placed, ref.lp_placed)


def test_prio_ragged_tasks_and_unaligned_outputs():
    lens = [0, 1, 2, 3, 7, 8, 9, 15, 16, 17, 31, 33, 63, 64, 65, 100, 127, 129, 255, 257, 500, 1000, 1001, 2047,
            0, 5, 6, 40, 41, 42, 43, 44] + [11 * k + 1 for k in range(32)]
    rec, off = ragged_trace(4242, lens, 9)
    prof, d_off, o_prof = check_profile(rec, off)
    rng = np.random.default_rng(5)
    for k_max in (2, 4, 9):
        hp, lo, lt, lq = prio_lists(rng, len(lens), 1500, k_max, same_level=0.7)
        check_prio(prof, d_off, off, o_prof, hp, lo, lt, lq, 300, 0)
        check_prio(prof, d_off, off, o_prof, hp, lo, lt, lq, 0, 5000)
    n_gaps = int(traces.gap_offsets(off, hp)[-1])
    out = binding.PrioFill(torch.empty(n_gaps + 1, dtype=torch.int32, device=DEV)[1:],
                           torch.empty(n_gaps + 1, dtype=torch.int64, device=DEV)[1:],
                           torch.empty(lt.size, dtype=torch.int64, device=DEV), torch.empty(lt.size, dtype=torch.int64, device=DEV))
    check_prio(prof, d_off, off, o_prof, hp, lo, lt, lq, 300, 0, out=out)


def test_prio_mixed_task_shapes():
    rec, off, _ = mixed_trace(99, 48, 6000, wide=False)
    prof, d_off, o_prof = check_profile(rec, off)
    rng = np.random.default_rng(8)
    for k_max in (3, 4, 16):
        hp, lo, lt, lq = prio_lists(rng, off.size - 1, 600, k_max)
        check_prio(prof, d_off, off, o_prof, hp, lo, lt, lq, 0, 0)
        check_prio(prof, d_off, off, o_prof, hp, lo, lt, lq, 2000, 20000)


def test_prio_argument_errors():
    cfg = traces.config(0)
    rec, off = traces.build(cfg)
    prof, d_off, o_prof = check_profile(rec, off)
    n_tasks = off.size - 1
    hp = np.zeros(2, dtype=np.uint32)
    go = binding.to_device_u64(traces.gap_offsets(off, hp), DEV)

    def call(lo, lt, lq, hp_=hp):
        return binding.fikit_prio_fill(prof.ids, d_off, prof.rows, prof.task_row_offsets, binding.to_device_u32(hp_, DEV),
                                       binding.to_device_u64(np.array(lo, dtype=np.uint64), DEV),
                                       binding.to_device_u32(np.array(lt, dtype=np.uint32), DEV),
                                       binding.to_device_u32(np.array(lq, dtype=np.uint32), DEV), go, margin_ns=0, min_gap_ns=0)

    call([0, 1, 2], [0, 1 % n_tasks], [1, 9])
    call([0, 0, 0], [], [])                                 # no low-priority task at all: every gap gets zeros
    for lo, lt, lq, status in (([0, 1, 2], [0, 0], [0, 1], binding.FIKIT_INVALID_ARG),       # level 0 is the high-priority task's
                               ([0, 1, 2], [0, 0], [1, 10], binding.FIKIT_INVALID_ARG),
                               ([0, 2, 1], [0, 0], [1, 1], binding.FIKIT_INVALID_ARG),       # offsets go down
                               ([1, 1, 2], [0, 0], [1, 1], binding.FIKIT_INVALID_ARG),       # first offset not 0
                               ([0, 1, 2], [0, n_tasks], [1, 1], binding.FIKIT_INVALID_ARG)):
        with pytest.raises(binding.FikitError) as e:
            call(lo, lt, lq)
        assert e.value.status == status, (lo, lq)
    with pytest.raises(binding.FikitError) as e:
        call([0, 1, 2], [0, 0], [1, 1], hp_=np.array([0, n_tasks], dtype=np.uint32))
    assert e.value.status == binding.FIKIT_INVALID_ARG
    out = call([0, 64, 64], [0] * 64, [5] * 64)             # the most the group kernels take
    torch.cuda.synchronize()
    assert out.lp_placed.numel() == 64


def test_prio_predictions_beyond_32_bits():
    """A prediction of 2^32 - 1 ns or more: the 64-bit kernels take the call; results are the oracle's."""
    lens = [40 + k for k in range(8)]
    rec, off = ragged_trace(5, lens, 4)
    slow = rec["name_id"] == 1
    ex = (rec["end_ns"] - rec["start_ns"]).astype(np.int64)
    ex[slow] += 5_000_000_000                       # a prediction that does not fit 32 bits
    gap = np.where(rec["name_id"] == 2, 11_000_000_000, 1000)              # and a kernel whose idle time such kernels fit into
    start = np.cumsum(ex + gap) - (ex + gap)
    rec["start_ns"], rec["end_ns"] = start, start + ex
    prof, d_off, o_prof = check_profile(rec, off)
    rng = np.random.default_rng(3)
    for k_max in (1, 3, 9):
        hp, lo, lt, lq = prio_lists(rng, off.size - 1, 12, k_max)
        for margin, min_gap in ((0, 0), (500, 2000)):
            got, exp = check_prio(prof, d_off, off, o_prof, hp, lo, lt, lq, margin, min_gap)
    assert int(exp[1].max()) > 2**32                 # (some gap did take more than 32 bits' worth)


@pytest.mark.parametrize("k", [65, 66, 130, 700])
def test_prio_more_tasks_in_a_scenario_than_a_wave_has_lanes(k):
    cfg = traces.config(4, n_tasks=24, hp_launches=300, lp_launches=90)
    rec, off = traces.build(cfg)
    prof, d_off, o_prof = check_profile(rec, off)
    rng = np.random.default_rng(k)
    n_scen = 5
    hp = rng.integers(0, cfg.n_tasks, n_scen).astype(np.uint32)
    counts = np.array([k, 3, 0, k - 1, 64][:n_scen])
    lo = np.zeros(n_scen + 1, dtype=np.uint64)
    np.cumsum(counts, out=lo[1:])
    lt = rng.integers(0, cfg.n_tasks, int(lo[-1])).astype(np.uint32)
    lq = rng.integers(1, 10, int(lo[-1])).astype(np.uint32)
    lq[rng.random(lq.shape[0]) < 0.6] = 2                      # many on one level: durations and ages decide
    got, exp = check_prio(prof, d_off, off, o_prof, hp, lo, lt, lq, cfg.margin_ns, cfg.min_gap_ns)
    assert int(exp[2].sum()) > 0


@pytest.mark.parametrize("seed", range(10))
def test_prio_seeded_sweep(seed):
    """Random task shapes, list lengths around the group-width borders, margins and thresholds."""
    rng = np.random.default_rng(1000 + seed)
    rec, off, _ = mixed_trace(300 + seed, 20, 4097, wide=False)
    prof, d_off, o_prof = check_profile(rec, off)
    for _ in range(3):
        k_max = int(rng.choice([1, 2, 3, 4, 5, 8, 9, 16, 17, 32, 33, 64]))
        n_scen = int(rng.integers(1, 400)) if k_max <= 9 else int(rng.integers(1, 40))
        hp, lo, lt, lq = prio_lists(rng, off.size - 1, n_scen, k_max, same_level=float(rng.choice([0.0, 0.5, 1.0])))
        margin = int(rng.choice([0, 1, 500, 10**6]))
        min_gap = int(rng.choice([0, 3, 10**4, 10**9]))
        predictor = int(rng.integers(0, 2))
        print(f"seed {seed}: up to {k_max} tasks, {n_scen} scenarios, margin {margin}, min gap {min_gap}, predictor {predictor}",
              flush=True)
        check_prio(prof, d_off, off, o_prof, hp, lo, lt, lq, margin, min_gap, predictor=predictor)
