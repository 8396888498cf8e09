"""Shared helpers of the GPU parity tests: run the HIP library and the CPU oracle on the same
seeded inputs and compare every output bit for bit."""
import numpy as np
import torch

import oracle
from paper_2311_10359_amd import binding, traces

DEV = "cuda:0"


def run_profile_gpu(rec, off, **kw):
    d_rec = binding.to_device_records(rec, DEV)
    d_off = binding.to_device_u64(off, DEV)
    prof = binding.fikit_profile(d_rec, d_off, **kw)
    torch.cuda.synchronize()
    return prof, d_off


def assert_profile_equal(prof, o_ids, o_rows, o_tro):
    ids = binding.u64_to_numpy(prof.ids)
    assert np.array_equal(ids, o_ids), "kernel IDs differ"
    assert prof.n_rows == len(o_rows), f"row count {prof.n_rows} != {len(o_rows)}"
    tro = binding.u64_to_numpy(prof.task_row_offsets)
    assert np.array_equal(tro, o_tro), "task row offsets differ"
    rows = binding.rows_to_numpy(prof.rows)
    if rows.tobytes() != o_rows.tobytes():
        for f in ("kernel_id", "task"):
            bad = np.nonzero(rows[f] != o_rows[f])[0]
            assert bad.size == 0, f"rows differ in {f} at {bad[:5]}"
        for blk in ("exec", "gap"):
            for f in ("count", "sum", "min", "max", "p50", "p95"):
                bad = np.nonzero(rows[blk][f] != o_rows[blk][f])[0]
                assert bad.size == 0, (f"rows differ in {blk}.{f} at {bad[:5]}: "
                                       f"{rows[blk][f][bad[:5]]} vs {o_rows[blk][f][bad[:5]]}")
        raise AssertionError("rows differ in reserved bytes")


def check_profile(rec, off, **kw):
    o_ids, o_rows, o_tro = oracle.profile(rec, off)
    prof, d_off = run_profile_gpu(rec, off, **kw)
    assert_profile_equal(prof, o_ids, o_rows, o_tro)
    return prof, d_off, (o_ids, o_rows, o_tro)


def check_gapfill(prof, d_off, off, o_prof, hp, lp, margin, min_gap, predictor=0):
    o_ids, o_rows, o_tro = o_prof
    go = traces.gap_offsets(off, hp)
    exp = oracle.gapfill(o_ids, off, o_rows, o_tro, hp, lp, margin, min_gap, go, predictor=predictor)
    got = binding.fikit_gapfill(prof.ids, d_off, prof.rows, prof.task_row_offsets,
                                binding.to_device_u32(hp, DEV), binding.to_device_u32(lp, DEV),
                                binding.to_device_u64(go, DEV), margin_ns=margin, min_gap_ns=min_gap, predictor=predictor)
    torch.cuda.synchronize()
    fc = binding.u32_to_numpy(got.fill_count)
    fn = got.filled_ns.cpu().numpy()
    comp = got.lp_completion_ns.cpu().numpy()
    placed = binding.u64_to_numpy(got.lp_placed)
    assert np.array_equal(placed, exp[3]), f"lp_placed differs: {placed[:8]} vs {exp[3][:8]}"
    bad = np.nonzero(fc != exp[0])[0]
    assert bad.size == 0, f"fill_count differs at {bad[:5]}: {fc[bad[:5]]} vs {exp[0][bad[:5]]}"
    bad = np.nonzero(fn != exp[1])[0]
    assert bad.size == 0, f"filled_ns differs at {bad[:5]}"
    assert np.array_equal(comp, exp[2]), f"lp_completion_ns differs: {comp[:8]} vs {exp[2][:8]}"
    return got
