"""Best low-priority partner per high-priority task: HIP library vs CPU oracle, element by element, through the
C ABI (needs an MI355X)."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2311_10359_amd import binding, traces
from parity_util import DEV, check_gapfill, check_profile
from test_oracle_pins import pairing_golden, random_pairing

pytestmark = pytest.mark.gpu


def run_pairing(hp, lp, n_tasks, go, fn, comp):
    got = binding.fikit_pairing_best(binding.to_device_u32(hp, DEV), binding.to_device_u32(lp, DEV), n_tasks,
                                     binding.to_device_u64(go, DEV), torch.from_numpy(fn).to(DEV), torch.from_numpy(comp).to(DEV))
    torch.cuda.synchronize()
    return (got.scenario_filled_ns.cpu().numpy(), binding.u64_to_numpy(got.best_scenario), binding.u32_to_numpy(got.best_lp),
            got.best_filled_ns.cpu().numpy())


def check_pairing(hp, lp, n_tasks, go, fn, comp):
    exp = oracle.pairing_best(hp, lp, n_tasks, go, fn, comp)
    got = run_pairing(hp, lp, n_tasks, go, fn, comp)
    for name, a, b in zip(("scenario_filled_ns", "best_scenario", "best_lp", "best_filled_ns"), got, exp):
        bad = np.nonzero(a != b)[0]
        assert bad.size == 0, f"{name} differs at {bad[:5]}: {a[bad[:5]]} vs {b[bad[:5]]}"


def test_pairing_hand_worked(golden_dir):
    with open(os.path.join(golden_dir, "p8_pairing_hand_worked.json")) as f:
        golden = json.load(f)
    hp, lp, n_tasks, go, fn, comp, exp = pairing_golden(golden)
    for a, b in zip(run_pairing(hp, lp, n_tasks, go, fn, comp), exp):
        assert np.array_equal(a, b)


def test_pairing_random_inputs_with_many_ties():
    rng = np.random.default_rng(18)
    for n_tasks, n_scen, max_gaps, values in ((1, 1, 0, 1), (7, 200, 3, 2), (50, 40, 9, 1000), (9, 3000, 2, 3),
                                              (300, 5000, 40, 10**12), (5, 300, 5000, 10**9), (40000, 70000, 1, 5)):
        hp, lp, go, fn, comp = random_pairing(rng, n_tasks, n_scen, max_gaps, values)
        print(f"{n_tasks} tasks, {n_scen} scenarios, {fn.size} gaps", flush=True)
        check_pairing(hp, lp, n_tasks, go, fn, comp)
    # no scenario at all
    got = run_pairing(np.zeros(0, np.uint32), np.zeros(0, np.uint32), 3, np.zeros(1, np.uint64), np.zeros(0, np.int64),
                      np.zeros(0, np.int64))
    assert got[0].size == 0 and (got[1] == np.uint64(2**64 - 1)).all() and (got[2] == np.uint32(2**32 - 1)).all()
    assert (got[3] == 0).all()


def test_pairing_of_a_grid_of_gap_fills():
    cfg = traces.config(1, n_tasks=24, launches=4000)          # 12 x 12 combinations
    rec, off = traces.build(cfg, threads=4)
    prof, d_off, o_prof = check_profile(rec, off)
    hp, lp = traces.scenarios(cfg)
    go = traces.gap_offsets(off, hp)
    got = check_gapfill(prof, d_off, off, o_prof, hp, lp, cfg.margin_ns, cfg.min_gap_ns)
    pair = binding.fikit_pairing_best(binding.to_device_u32(hp, DEV), binding.to_device_u32(lp, DEV), cfg.n_tasks,
                                      binding.to_device_u64(go, DEV), got.filled_ns, got.lp_completion_ns)
    torch.cuda.synchronize()
    o_ids, o_rows, o_tro = o_prof
    o_fill = oracle.gapfill(o_ids, off, o_rows, o_tro, hp, lp, cfg.margin_ns, cfg.min_gap_ns, go)
    exp = oracle.pairing_best(hp, lp, cfg.n_tasks, go, o_fill[1], o_fill[2])
    assert np.array_equal(pair.scenario_filled_ns.cpu().numpy(), exp[0])
    assert np.array_equal(binding.u64_to_numpy(pair.best_scenario), exp[1])
    assert np.array_equal(binding.u32_to_numpy(pair.best_lp), exp[2])
    assert np.array_equal(pair.best_filled_ns.cpu().numpy(), exp[3])
    assert (exp[2][:12] >= 12).all() and (exp[2][12:] == np.uint32(2**32 - 1)).all()


def test_pairing_argument_errors():
    hp, lp = np.array([0, 1], np.uint32), np.array([1, 0], np.uint32)
    fn, comp = np.arange(5, dtype=np.int64), np.array([1, 2], np.int64)
    for bad_hp, bad_go in ((np.array([0, 2], np.uint32), [0, 2, 5]), (hp, [0, 3, 2]), (hp, [1, 2, 5]), (hp, [0, 6, 5])):
        with pytest.raises(binding.FikitError) as e:
            run_pairing(bad_hp, lp, 2, np.array(bad_go, np.uint64), fn, comp)
        assert e.value.status == binding.FIKIT_INVALID_ARG, bad_go
    run_pairing(hp, lp, 2, np.array([0, 2, 5], np.uint64), fn, comp)
