"""The five workloads at their full sizes, in the launch configuration bench.py times.

fikit_profile and fikit_gapfill are compared with the oracle whole: every Kernel ID, every row, every
gap and every scenario (worker processes regenerate the workload piece by piece from its seeds and run
the single-threaded oracle on each piece, see whole_workload.py).  The calls that build on them (replay,
priority queues, pairing, merge, measurement) are checked at full size on sampled scenarios recomputed
one by one, plus properties that hold at any size."""
import time

import numpy as np
import pytest
import torch

import oracle
from paper_2311_10359_amd import binding, traces
from parity_util import DEV
from whole_workload import compare_whole_workload

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


def upload(cfg, workers=16):
    off = traces.task_offsets(cfg)
    n = int(off[-1])
    d_rec = torch.empty((n, 64), dtype=torch.uint8, device=DEV)
    t0 = time.time()
    last = t0
    for first, view in traces.stream(cfg, workers=workers):
        u8 = view.view(np.uint8).reshape(-1, 64)
        d_rec[first:first + u8.shape[0]].copy_(torch.from_numpy(u8))
        if time.time() - last > 15:
            last = time.time()
            say(f"  uploading ... {time.time() - t0:.0f}s")
    torch.cuda.synchronize()
    say(f"  {n} records resident after {time.time() - t0:.1f}s")
    return d_rec, off


def check_global_properties(prof, off, n_tasks):
    rows = prof.rows.view(torch.int64).reshape(-1, 16)      # 16 eight-byte fields per row
    n = int(off[-1])
    nonempty = int(np.count_nonzero(off[1:] > off[:-1]))
    assert int(rows[:, 2].sum()) == n                      # exec.count
    assert int(rows[:, 8].sum()) == n - nonempty           # gap.count
    for base in (2, 8):
        cnt, mn, mx, p50, p95 = rows[:, base], rows[:, base + 2], rows[:, base + 3], rows[:, base + 4], rows[:, base + 5]
        has = cnt > 0
        assert bool(((mn <= p50) & (p50 <= p95) & (p95 <= mx) & (mn >= 0))[has].all())
        assert bool((rows[:, base + 1:base + 6][~has] == 0).all())
    task = rows[:, 1] & 0xffffffff
    tro = prof.task_row_offsets
    assert int(tro[0]) == 0 and int(tro[-1]) == prof.n_rows
    assert bool((tro[1:] >= tro[:-1]).all())
    # rows are grouped by task in order, IDs strictly ascending (unsigned) inside a task
    assert bool((task[1:] >= task[:-1]).all())
    same = task[1:] == task[:-1]
    kid = rows[:, 0]
    flip = torch.tensor(-2 ** 63, dtype=torch.int64, device=kid.device)
    ukey = kid ^ flip                                       # unsigned order as signed order
    assert bool((ukey[1:] > ukey[:-1])[same].all())
    expect_task = torch.repeat_interleave(torch.arange(n_tasks, device=kid.device), tro[1:] - tro[:-1])
    assert torch.equal(task, expect_task)


def profile_full(cfg):
    d_rec, off = upload(cfg)
    d_off = binding.to_device_u64(off, DEV)
    row_cap = sum(cfg.ids(t) for t in range(cfg.n_tasks))
    t0 = time.time()
    prof = binding.fikit_profile(d_rec, d_off, row_capacity=row_cap)
    say(f"  fikit_profile: {prof.n_rows} rows in {time.time() - t0:.2f}s")
    return prof, off, d_off, d_rec


def test_config1_medium_full_oracle():
    cfg = traces.config(1)
    say("config 1 (medium), whole workload against the oracle")
    rec, off = traces.build(cfg, threads=8)
    o_ids, o_rows, o_tro = oracle.profile(rec, off)
    d_off = binding.to_device_u64(off, DEV)
    prof = binding.fikit_profile(binding.to_device_records(rec, DEV), d_off)
    assert np.array_equal(binding.u64_to_numpy(prof.ids), o_ids)
    assert binding.rows_to_numpy(prof.rows).tobytes() == o_rows.tobytes()
    assert np.array_equal(binding.u64_to_numpy(prof.task_row_offsets), o_tro)
    check_global_properties(prof, off, cfg.n_tasks)
    hp, lp = traces.scenarios(cfg)
    go = traces.gap_offsets(off, hp)
    exp = oracle.gapfill(o_ids, off, o_rows, o_tro, hp, lp, cfg.margin_ns, cfg.min_gap_ns, go)
    got = binding.fikit_gapfill(prof.ids, d_off, prof.rows, prof.task_row_offsets, binding.to_device_u32(hp, DEV),
                                binding.to_device_u32(lp, DEV), binding.to_device_u64(go, DEV),
                                margin_ns=cfg.margin_ns, min_gap_ns=cfg.min_gap_ns)
    assert np.array_equal(binding.u32_to_numpy(got.fill_count), exp[0])
    assert np.array_equal(got.filled_ns.cpu().numpy(), exp[1])
    assert np.array_equal(got.lp_completion_ns.cpu().numpy(), exp[2])
    assert np.array_equal(binding.u64_to_numpy(got.lp_placed), exp[3])


@pytest.mark.parametrize("index", [2, 3])
def test_profile_only_workloads_full_size(index):
    cfg = traces.config(index)
    say(f"config {index} ({cfg.name}), {cfg.n_records} records, whole workload against the oracle")
    prof, off, d_off, d_rec = profile_full(cfg)
    del d_rec
    check_global_properties(prof, off, cfg.n_tasks)
    compare_whole_workload(cfg, off, {"ids": prof.ids, "rows": prof.rows, "task_row_offsets": prof.task_row_offsets}, say=say)


def test_config4_one_call_full_size():
    """The benchmark's default step: fikit_profile_gapfill over the whole workload, every output against the oracle."""
    cfg = traces.config(4)
    say(f"config 4 ({cfg.name}), {cfg.n_records} records, profile and gap fill as one call")
    d_rec, off = upload(cfg)
    d_off = binding.to_device_u64(off, DEV)
    hp, lp = traces.scenarios(cfg)
    go = traces.gap_offsets(off, hp)
    d_go = binding.to_device_u64(go, DEV)
    row_cap = sum(cfg.ids(t) for t in range(cfg.n_tasks))
    t0 = time.time()
    prof, got = binding.fikit_profile_gapfill(d_rec, d_off, binding.to_device_u32(hp, DEV), binding.to_device_u32(lp, DEV), d_go,
                                              margin_ns=cfg.margin_ns, min_gap_ns=cfg.min_gap_ns, row_capacity=row_cap)
    torch.cuda.synchronize()
    say(f"  fikit_profile_gapfill: {prof.n_rows} rows, {hp.size} scenarios in {time.time() - t0:.2f}s")
    del d_rec
    check_global_properties(prof, off, cfg.n_tasks)
    whole = compare_whole_workload(cfg, off, {"ids": prof.ids, "rows": prof.rows, "task_row_offsets": prof.task_row_offsets,
                                              "gap_offsets": d_go, "fill_count": got.fill_count, "filled_ns": got.filled_ns,
                                              "lp_completion_ns": got.lp_completion_ns, "lp_placed": got.lp_placed}, say=say)
    assert whole["equal_scenarios"] == hp.size and whole["equal_tasks"] == cfg.n_tasks


def test_config4_batched_gapfill_full_size():
    cfg = traces.config(4)
    say(f"config 4 ({cfg.name}), {cfg.n_records} records")
    prof, off, d_off, d_rec = profile_full(cfg)
    check_global_properties(prof, off, cfg.n_tasks)
    scen = [0, 1, 777, 32768, 65534, 65535]
    # the profile merged with itself: same IDs, counts and sums doubled (modulo 2^64), everything else as it was
    twice = binding.fikit_profile_merge(prof.rows, prof.task_row_offsets, prof.rows, prof.task_row_offsets)
    torch.cuda.synchronize()
    assert twice.n_rows == prof.n_rows and torch.equal(twice.task_row_offsets, prof.task_row_offsets)
    r1, r2 = prof.rows.view(torch.int64).reshape(-1, 16), twice.rows.view(torch.int64).reshape(-1, 16)
    doubled = [2, 3, 8, 9]                                   # exec.count, exec.sum, gap.count, gap.sum
    same = [f for f in range(16) if f not in doubled]
    assert torch.equal(r2[:, same], r1[:, same]) and torch.equal(r2[:, doubled], r1[:, doubled] * 2)
    say("  fikit_profile_merge of the profile with itself: consistent at full size")
    del twice, r1, r2
    # per-launch measurement at full size (the actual idle times are the replay's input further down)
    d_exec, d_gap = binding.fikit_measure(d_rec, d_off)
    for s in scen[:3]:
        for t in (2 * s, 2 * s + 1):
            rec_t = traces.task_records(cfg, t)
            ex, gp = oracle.measure(rec_t, np.array([0, rec_t.shape[0]], dtype=np.uint64))
            a, b = int(off[t]), int(off[t + 1])
            assert np.array_equal(d_exec[a:b].cpu().numpy(), ex) and np.array_equal(d_gap[a:b].cpu().numpy(), gp), f"task {t}"
    assert bool((d_exec >= 1).all())
    del d_rec, d_exec
    hp, lp = traces.scenarios(cfg)
    go = traces.gap_offsets(off, hp)
    t0 = time.time()
    got = binding.fikit_gapfill(prof.ids, d_off, prof.rows, prof.task_row_offsets, binding.to_device_u32(hp, DEV),
                                binding.to_device_u32(lp, DEV), binding.to_device_u64(go, DEV),
                                margin_ns=cfg.margin_ns, min_gap_ns=cfg.min_gap_ns)
    say(f"  fikit_gapfill: {hp.size} scenarios in {time.time() - t0:.2f}s")
    # properties at full size: per scenario, the per-gap counts add up to the number placed
    fc = got.fill_count.view(-1, 4095).to(torch.int64)
    placed = got.lp_placed
    assert torch.equal(fc.sum(dim=1), placed)
    assert bool((placed <= 16384).all()) and bool((got.filled_ns >= 0).all())
    assert bool((got.lp_completion_ns > 0).all())
    # the whole workload against the oracle: every task's IDs and rows, every scenario's outputs
    d_hp, d_lp, d_go = binding.to_device_u32(hp, DEV), binding.to_device_u32(lp, DEV), binding.to_device_u64(go, DEV)
    whole = compare_whole_workload(cfg, off, {"ids": prof.ids, "rows": prof.rows, "task_row_offsets": prof.task_row_offsets,
                                              "gap_offsets": d_go, "fill_count": got.fill_count, "filled_ns": got.filled_ns,
                                              "lp_completion_ns": got.lp_completion_ns, "lp_placed": got.lp_placed}, say=say)
    assert whole["equal_scenarios"] == hp.size
    # best partner per high-priority task over these results: every task heads exactly one scenario here, so the
    # search must return that scenario, and the per-scenario sums must be the row sums of the filled times
    pair = binding.fikit_pairing_best(d_hp, d_lp, cfg.n_tasks, d_go, got.filled_ns, got.lp_completion_ns)
    torch.cuda.synchronize()
    assert torch.equal(pair.scenario_filled_ns, got.filled_ns.view(-1, 4095).sum(dim=1))
    heads = torch.from_numpy(hp.astype(np.int64)).to(DEV)
    assert torch.equal(pair.best_scenario[heads], torch.arange(hp.size, device=DEV))
    assert torch.equal(pair.best_lp[heads].to(torch.int64), torch.from_numpy(lp.astype(np.int64)).to(DEV))
    assert torch.equal(pair.best_filled_ns[heads], pair.scenario_filled_ns)
    others = torch.ones(cfg.n_tasks, dtype=torch.bool, device=DEV)
    others[heads] = False
    assert bool((pair.best_scenario[others] == -1).all()) and bool((pair.best_lp[others] == -1).all())
    assert bool((pair.best_filled_ns[others] == 0).all())
    say("  fikit_pairing_best: sums and picks consistent at full size")
    del pair
    # replay against the actual idle times, without and with real-time feedback
    hp_gap = d_gap.view(-1, 4096 + 16384)[:, :4095]          # actual idle time of every gap, scenario by scenario
    for feedback in (False, True):
        t0 = time.time()
        rep = binding.fikit_gapfill_replay(prof.ids, d_off, prof.rows, prof.task_row_offsets, d_gap, d_hp, d_lp, d_go,
                                           margin_ns=cfg.margin_ns, min_gap_ns=cfg.min_gap_ns, feedback=feedback)
        say(f"  fikit_gapfill_replay(feedback={feedback}): {hp.size} scenarios in {time.time() - t0:.2f}s")
        fn = rep.filled_ns.view(-1, 4095)
        assert torch.equal(rep.fill_count.view(-1, 4095).to(torch.int64).sum(dim=1), rep.lp_placed)
        assert torch.equal(torch.clamp(fn - hp_gap, min=0).sum(dim=1), rep.hp_delay_ns)
        if not feedback:   # the profile-only controller takes the decisions of the gap fill
            assert torch.equal(rep.fill_count, got.fill_count) and torch.equal(rep.filled_ns, got.filled_ns)
            assert torch.equal(rep.lp_placed, got.lp_placed)
        for s in scen:
            recs = [traces.task_records(cfg, 2 * s), traces.task_records(cfg, 2 * s + 1)]
            loc_off = np.array([0, recs[0].shape[0], recs[0].shape[0] + recs[1].shape[0]], dtype=np.uint64)
            both = np.concatenate(recs)
            o_ids, o_rows, o_tro = oracle.profile(both, loc_off)
            _, o_gap = oracle.measure(both, loc_off)
            one = np.array([0], dtype=np.uint32)
            exp = oracle.replay(o_ids, loc_off, o_rows, o_tro, o_gap, one, one + 1, cfg.margin_ns, cfg.min_gap_ns, feedback,
                                traces.gap_offsets(loc_off, one))
            g0, g1 = int(go[s]), int(go[s + 1])
            assert np.array_equal(binding.u32_to_numpy(rep.fill_count[g0:g1]), exp[0]), f"scenario {s}"
            assert np.array_equal(rep.filled_ns[g0:g1].cpu().numpy(), exp[1]), f"scenario {s}"
            assert int(rep.hp_delay_ns[s]) == int(exp[2][0]) and int(rep.lp_placed[s]) == int(exp[3][0])
        say(f"  replay, feedback={feedback}: mean delay of the high-priority task {float(rep.hp_delay_ns.double().mean()) / 1e6:.3f} ms; "
            f"sampled scenarios match the oracle")
        del rep
    del d_gap, got
    # three low-priority tasks per scenario in priority queues (the configuration bench.py --prio 3 times)
    k = 3
    _, p_lo, p_lt, p_lq = traces.prio_scenarios(cfg, k)
    t0 = time.time()
    pf = binding.fikit_prio_fill(prof.ids, d_off, prof.rows, prof.task_row_offsets, d_hp, binding.to_device_u64(p_lo, DEV),
                                 binding.to_device_u32(p_lt, DEV), binding.to_device_u32(p_lq, DEV), d_go,
                                 margin_ns=cfg.margin_ns, min_gap_ns=cfg.min_gap_ns)
    say(f"  fikit_prio_fill: {hp.size} scenarios with {k} low-priority tasks each in {time.time() - t0:.2f}s")
    # properties at full size: what the gaps of a scenario took is what its tasks placed
    assert torch.equal(pf.fill_count.view(-1, 4095).to(torch.int64).sum(dim=1), pf.lp_placed.view(-1, k).sum(dim=1))
    assert torch.equal(pf.filled_ns.view(-1, 4095).sum(dim=1), pf.lp_placed_ns.view(-1, k).sum(dim=1))
    assert bool((pf.lp_placed <= 16384).all()) and bool((pf.filled_ns >= 0).all())
    for s in scen:
        tasks = [2 * s] + [int(t) for t in p_lt[k * s:k * s + k]]
        recs = [traces.task_records(cfg, t) for t in tasks]
        loc_off = np.zeros(len(recs) + 1, dtype=np.uint64)
        np.cumsum([r.shape[0] for r in recs], out=loc_off[1:])
        o_ids, o_rows, o_tro = oracle.profile(np.concatenate(recs), loc_off)
        one = np.array([0], dtype=np.uint32)
        exp = oracle.prio_fill(o_ids, loc_off, o_rows, o_tro, one, np.array([0, k], dtype=np.uint64),
                               np.arange(1, k + 1, dtype=np.uint32), p_lq[k * s:k * s + k], cfg.margin_ns, cfg.min_gap_ns,
                               traces.gap_offsets(loc_off, one))
        g0, g1 = int(go[s]), int(go[s + 1])
        assert np.array_equal(binding.u32_to_numpy(pf.fill_count[g0:g1]), exp[0]), f"scenario {s}"
        assert np.array_equal(pf.filled_ns[g0:g1].cpu().numpy(), exp[1]), f"scenario {s}"
        assert np.array_equal(binding.u64_to_numpy(pf.lp_placed[k * s:k * s + k]), exp[2]), f"scenario {s}"
        assert np.array_equal(pf.lp_placed_ns[k * s:k * s + k].cpu().numpy(), exp[3]), f"scenario {s}"
    say(f"  priority queues: sampled scenarios {scen} match the oracle")
