"""The whole-workload checker itself (host logic, no GPU): fed the oracle's own outputs it must find every
task and scenario equal; one flipped element anywhere must be found and named."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_10359_amd import traces
from whole_workload import compare_whole_workload


def oracle_outputs(cfg):
    rec, off = traces.build(cfg)
    ids, rows, tro = oracle.profile(rec, off)
    out = {"ids": torch.from_numpy(ids.view(np.int64).copy()),
           "rows": torch.from_numpy(rows.view(np.uint8).reshape(-1, 128).copy()),
           "task_row_offsets": torch.from_numpy(tro.view(np.int64).copy())}
    hp, lp = traces.scenarios(cfg)
    if hp.size:
        go = traces.gap_offsets(off, hp)
        fc, fn, comp, placed = oracle.gapfill(ids, off, rows, tro, hp, lp, cfg.margin_ns, cfg.min_gap_ns, go)
        out.update({"gap_offsets": torch.from_numpy(go.view(np.int64).copy()), "fill_count": torch.from_numpy(fc.view(np.int32).copy()),
                    "filled_ns": torch.from_numpy(fn.copy()), "lp_completion_ns": torch.from_numpy(comp.copy()),
                    "lp_placed": torch.from_numpy(placed.view(np.int64).copy())})
    return off, out


def quiet(_):
    pass


def test_checker_accepts_equal_outputs_and_counts_everything():
    cfg = traces.config(4, n_tasks=24, hp_launches=300, lp_launches=900)
    off, out = oracle_outputs(cfg)
    total = compare_whole_workload(cfg, off, out, records_per_piece=3000, workers=2, say=quiet)
    assert total["equal_tasks"] == 24 and total["equal_scenarios"] == 12
    cfg = traces.config(3, n_tasks=5, launches=3000)
    off, out = oracle_outputs(cfg)
    total = compare_whole_workload(cfg, off, out, records_per_piece=3000, workers=2, say=quiet)
    assert total["equal_tasks"] == 5 and total["scenarios"] == 0


@pytest.mark.parametrize("name,at", [("ids", 2500), ("rows", 128 * 700 + 40), ("fill_count", 1234), ("filled_ns", 3000),
                                     ("lp_completion_ns", 11), ("lp_placed", 0), ("task_row_offsets", 7)])
def test_checker_finds_one_flipped_element(name, at):
    cfg = traces.config(4, n_tasks=24, hp_launches=300, lp_launches=900)
    off, out = oracle_outputs(cfg)
    flat = out[name].view(-1)
    flat[at] = flat[at] + 1
    with pytest.raises(AssertionError, match="differ"):
        compare_whole_workload(cfg, off, out, records_per_piece=3000, workers=2, say=quiet)
