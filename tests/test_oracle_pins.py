"""Pins of the CPU oracle to things other than itself.

P0  published FNV-1a-64 vectors (kernel ID hash).
P1  hand-worked 12-launch trace (tests/golden/p1_hand_worked.json).
P2  the paper's closed forms SK_j, SG_j (Section 3.2) evaluated with the Kronecker delta as printed.
P3  invariants that hold for any trace.
P4  brute-force enumeration of every first-in-first-out schedule on tiny traces.
P5  special cases that reduce to library routines (numpy.sort, numpy.unique) or closed forms.
P6  per-launch measurement and the replay against actual idle times: hand-worked example
    (tests/golden/p6_replay_hand_worked.json), ties to the pinned gap fill, closed form by prefix sums.
P7  several low-priority tasks in priority queues (BestPrioFit): hand-worked cases after the paper's own example
    (tests/golden/p7_prio_fill_hand_worked.json), the one-task case against the pinned gap fill, and every
    decision of the issue log checked against the rule written as a sort key.
P8  best partner per high-priority task: a hand-worked case (tests/golden/p8_pairing_hand_worked.json), numpy's
    lexsort on random inputs, and the gap fill of a grid of combinations searched by a plain Python loop.
P9  profiles merged over runs: a hand-worked case (tests/golden/p9_merge_hand_worked.json), and the merge of the
    profiles of a task's runs against the profile of the whole trace with the idle times between runs taken out
    (count, sum, min, max; numpy on the pinned per-launch measurements), identity and symmetry.
"""
import itertools
import json
import os
import struct
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2311_10359_amd import traces

U64 = (1 << 64) - 1


def make_records(items):
    """items: list of (name_id, grid3, block3, shmem, start, end)."""
    rec = np.zeros(len(items), dtype=traces.LAUNCH_DTYPE)
    for i, (name, grid, block, shmem, start, end) in enumerate(items):
        rec[i]["name_id"] = name
        rec[i]["grid"] = grid
        rec[i]["block"] = block
        rec[i]["shmem"] = shmem
        rec[i]["start_ns"] = start
        rec[i]["end_ns"] = end
    return rec


def stats_tuple(s):
    return [int(s["count"]), int(s["sum"]), int(s["min"]), int(s["max"]), int(s["p50"]), int(s["p95"])]


# ---------------------------------------------------------------- P0
@pytest.mark.parametrize("data,expected", [
    (b"", 0xcbf29ce484222325),          # offset basis
    (b"a", 0xaf63dc4c8601ec8c),         # published FNV-1a 64 test vectors
    (b"foobar", 0x85944171f73967e8),
])
def test_p0_fnv1a64_published_vectors(data, expected):
    assert oracle.kernel_id(data) == expected


def test_p0_id_covers_exactly_the_identity_bytes():
    base = make_records([(5, (7, 8, 9), (10, 11, 12), 13, 100, 200)])
    ids0, _, _ = oracle.profile(base, np.array([0, 1], dtype=np.uint64))
    raw = base.tobytes()
    assert int(ids0[0]) == oracle.kernel_id(raw[:32])
    # timestamps and reserved bytes never enter the ID
    other = base.copy()
    other["start_ns"] = 1
    other["end_ns"] = 9
    other["reserved"] = 0xAB
    ids1, _, _ = oracle.profile(other, np.array([0, 1], dtype=np.uint64))
    assert ids1[0] == ids0[0]
    # every one of the eight identity fields does
    seen = {int(ids0[0])}
    for field, idx in [("name_id", None), ("grid", 0), ("grid", 1), ("grid", 2), ("block", 0),
                       ("block", 1), ("block", 2), ("shmem", None)]:
        m = base.copy()
        if idx is None:
            m[field] += 1
        else:
            m[field][0, idx] += 1
        ids2, _, _ = oracle.profile(m, np.array([0, 1], dtype=np.uint64))
        seen.add(int(ids2[0]))
    assert len(seen) == 9


# ---------------------------------------------------------------- P1
@pytest.fixture(scope="module")
def p1(golden_dir):
    with open(os.path.join(golden_dir, "p1_hand_worked.json")) as f:
        g = json.load(f)
    k = g["kernels"]

    def rec_of(trace):
        return make_records([(k[n]["name_id"], k[n]["grid"], k[n]["block"], k[n]["shmem"], s, e)
                             for n, s, e in trace])
    rec = np.concatenate([rec_of(g["hp_trace"]), rec_of(g["lp_trace"])])
    off = np.array([0, len(g["hp_trace"]), len(g["hp_trace"]) + len(g["lp_trace"])], dtype=np.uint64)
    return g, rec, off


def test_p1_ids_and_rows(p1):
    g, rec, off = p1
    ids, rows, tro = oracle.profile(rec, off)
    names = [n for n, _, _ in g["hp_trace"]] + [n for n, _, _ in g["lp_trace"]]
    for i, n in enumerate(names):
        assert int(ids[i]) == int(g["kernels"][n]["id"], 16)
    assert list(tro) == [0, 3, 5]
    assert len(rows) == 5
    for r, name in zip(rows, g["rows_in_order"]):
        exp = g["rows"][name]
        assert int(r["kernel_id"]) == int(g["kernels"][name]["id"], 16)
        assert int(r["task"]) == exp["task"]
        assert stats_tuple(r["exec"]) == exp["exec"]
        assert stats_tuple(r["gap"]) == exp["gap"]
    # the paper's means: SK_A = 21000, SG_C = 310000 / 3
    a = rows[1]
    c = rows[2]
    assert Fraction(int(a["exec"]["sum"]), int(a["exec"]["count"])) == g["paper_means"]["SK_A"]
    assert int(c["gap"]["sum"]) == g["paper_means"]["SG_C_times_3"] and int(c["gap"]["count"]) == 3
    assert sum(int(r["exec"]["count"]) for r in rows[:3]) == 12
    assert sum(int(r["gap"]["count"]) for r in rows[:3]) == 11


@pytest.mark.parametrize("case", [0, 1, 2])
def test_p1_gapfill(p1, case):
    g, rec, off = p1
    exp = g["gapfill"][case]
    ids, rows, tro = oracle.profile(rec, off)
    hp = np.array([0], dtype=np.uint32)
    lp = np.array([1], dtype=np.uint32)
    go = traces.gap_offsets(off, hp)
    assert list(go) == [0, 11]
    fc, fn, comp, placed, assign, aoff = oracle.gapfill(
        ids, off, rows, tro, hp, lp, exp["margin_ns"], exp["min_gap_ns"], go, want_assign=True,
        predictor=exp.get("predictor", 0))
    assert list(fc) == exp["fill_count"]
    assert list(fn) == exp["filled_ns"]
    assert int(placed[0]) == exp["lp_placed"]
    assert int(comp[0]) == exp["lp_completion_ns"]
    assert list(assign) == exp["assign"]


# ---------------------------------------------------------------- P2
def test_p2_paper_closed_forms_sk_sg():
    cfg = traces.config(0, launches=240)
    rec, off = traces.build(cfg)
    ids, rows, tro = oracle.profile(rec, off)
    for t in range(cfg.n_tasks):
        lo, hi = int(off[t]), int(off[t + 1])
        tid = [int(x) for x in ids[lo:hi]]
        K = [int(rec["end_ns"][i] - rec["start_ns"][i]) for i in range(lo, hi)]
        G = [max(0, int(rec["start_ns"][i + 1] - rec["end_ns"][i])) for i in range(lo, hi - 1)]
        s_uid = sorted(set(tid))
        assert [int(r["kernel_id"]) for r in rows[int(tro[t]):int(tro[t + 1])]] == s_uid
        for j, r in zip(s_uid, rows[int(tro[t]):int(tro[t + 1])]):
            num = sum(K[i] * (1 if tid[i] == j else 0) for i in range(len(K)))
            den = sum(1 * (1 if tid[i] == j else 0) for i in range(len(K)))
            assert Fraction(int(r["exec"]["sum"]), int(r["exec"]["count"])) == Fraction(num, den)
            numg = sum(G[i] * (1 if tid[i] == j else 0) for i in range(len(G)))
            deng = sum(1 * (1 if tid[i] == j else 0) for i in range(len(G)))
            assert int(r["gap"]["count"]) == deng and int(r["gap"]["sum"]) == numg


# ---------------------------------------------------------------- P3
def small_configs():
    return [
        traces.config(0),
        traces.config(1, n_tasks=4, launches=3000),
        traces.config(2, n_tasks=2, launches=20000),
        traces.config(3, n_tasks=3, launches=10000),
        traces.config(4, n_tasks=6, hp_launches=512, lp_launches=2048),
    ]


@pytest.mark.parametrize("cfg", small_configs(), ids=lambda c: c.name)
def test_p3_profile_invariants(cfg):
    rec, off = traces.build(cfg)
    ids, rows, tro = oracle.profile(rec, off)
    n = rec.shape[0]
    nonempty = int(np.count_nonzero(off[1:] > off[:-1]))
    assert int(rows["exec"]["count"].sum()) == n
    assert int(rows["gap"]["count"].sum()) == n - nonempty
    for blk in ("exec", "gap"):
        s = rows[blk]
        has = s["count"] > 0
        assert np.all(s["min"][has] <= s["p50"][has])
        assert np.all(s["p50"][has] <= s["p95"][has])
        assert np.all(s["p95"][has] <= s["max"][has])
        assert np.all(s["min"][has] >= 0)
        cnt = s["count"][has].astype(object)
        assert all(c * int(mn) <= int(sm) <= c * int(mx) for c, mn, sm, mx in
                   zip(cnt, s["min"][has], s["sum"][has], s["max"][has]))
        z = ~has
        for f in ("sum", "min", "max", "p50", "p95"):
            assert np.all(s[f][z] == 0)
    # rows strictly increasing in (task, id)
    key = list(zip(rows["task"].tolist(), rows["kernel_id"].tolist()))
    assert all(a < b for a, b in zip(key, key[1:]))
    for t in range(cfg.n_tasks):
        assert np.all(rows["task"][int(tro[t]):int(tro[t + 1])] == t)


def test_p3_exec_stats_do_not_depend_on_launch_order():
    # Section 3.2: the Kernel ID is independent of the kernel's position within the task.
    cfg = traces.config(1, n_tasks=2, launches=2000)
    rec, off = traces.build(cfg)
    _, rows, _ = oracle.profile(rec, off)
    rng = np.random.default_rng(7)
    perm = rec.copy()
    for t in range(cfg.n_tasks):
        lo, hi = int(off[t]), int(off[t + 1])
        perm[lo:hi] = rec[lo:hi][rng.permutation(hi - lo)]
    _, rows2, _ = oracle.profile(perm, off)
    assert np.array_equal(rows["kernel_id"], rows2["kernel_id"])
    assert np.array_equal(rows["exec"], rows2["exec"])


def test_p3_negative_idle_time_clamps_to_zero():
    rec = make_records([(1, (1, 1, 1), (1, 1, 1), 0, 0, 100),     # overlaps with the next
                        (1, (1, 1, 1), (1, 1, 1), 0, 50, 150),
                        (1, (1, 1, 1), (1, 1, 1), 0, 170, 180)])
    _, rows, _ = oracle.profile(rec, np.array([0, 3], dtype=np.uint64))
    assert stats_tuple(rows[0]["gap"]) == [2, 20, 0, 20, 0, 20]
    assert stats_tuple(rows[0]["exec"]) == [3, 210, 10, 100, 100, 100]


@pytest.mark.parametrize("cfg", [small_configs()[0], small_configs()[1], small_configs()[4]],
                         ids=lambda c: c.name)
@pytest.mark.parametrize("min_gap", [0, 100000])
def test_p3_gapfill_invariants(cfg, min_gap):
    rec, off = traces.build(cfg)
    ids, rows, tro = oracle.profile(rec, off)
    hp, lp = traces.scenarios(cfg)
    go = traces.gap_offsets(off, hp)
    margin = cfg.margin_ns
    fc, fn, comp, placed, assign, aoff = oracle.gapfill(ids, off, rows, tro, hp, lp, margin, min_gap, go,
                                                        want_assign=True)
    for s in range(hp.shape[0]):
        h0, h1 = int(off[hp[s]]), int(off[hp[s] + 1])
        l0, l1 = int(off[lp[s]]), int(off[lp[s] + 1])
        hr = rows[int(tro[hp[s]]):int(tro[hp[s] + 1])]
        lr = rows[int(tro[lp[s]]):int(tro[lp[s] + 1])]
        gp50 = dict(zip(hr["kernel_id"].tolist(), hr["gap"]["p50"].tolist()))
        ep50 = dict(zip(hr["kernel_id"].tolist(), hr["exec"]["p50"].tolist()))
        dp50 = dict(zip(lr["kernel_id"].tolist(), lr["exec"]["p50"].tolist()))
        G = np.array([gp50[i] for i in ids[h0:h1 - 1].tolist()], dtype=np.int64)
        D = np.array([dp50[i] for i in ids[l0:l1].tolist()], dtype=np.int64)
        f = fn[int(go[s]):int(go[s + 1])]
        c = fc[int(go[s]):int(go[s + 1])]
        a = assign[int(aoff[s]):int(aoff[s + 1])]
        assert np.all(f >= 0)
        assert np.all(f <= np.maximum(0, G - margin)) and np.all(f <= G)
        assert np.all(f[G < min_gap] == 0) and np.all(c[G < min_gap] == 0)
        assert int(c.sum()) == int(placed[s]) <= l1 - l0
        # first-in-first-out: the gap index is non-decreasing along the low-priority queue
        assert np.all(np.diff(a.astype(np.int64)) >= 0)
        p = int(placed[s])
        assert np.all(a[:p] != 0xffffffff) and np.all(a[p:] == 0xffffffff)
        assert np.array_equal(np.bincount(a[:p], minlength=c.shape[0])[:c.shape[0]], c)
        assert np.array_equal(np.bincount(a[:p], weights=D[:p], minlength=f.shape[0]).astype(np.int64), f)
        # completion can never precede doing all the low-priority work back to back
        assert int(comp[s]) >= int(D.sum())
        t_end = sum(ep50[i] for i in ids[h0:h1].tolist()) + int(G.sum())
        if p < l1 - l0:
            assert int(comp[s]) == t_end + int(D[p:].sum())
        else:
            assert int(comp[s]) <= t_end


# ---------------------------------------------------------------- P4
def tiny_scenario(rng, H, L, durations, gaps):
    """One HP task and one LP task whose every kernel ID occurs once, so p50 == the sample."""
    items = []
    t = 0
    for i in range(H):
        e = int(rng.choice([1000, 3000]))
        g = int(rng.choice(gaps))
        items.append((100 + i, (1, 1, 1), (64, 1, 1), 0, t, t + e))
        t += e + g
    hp_n = len(items)
    t = 0
    for j in range(L):
        d = int(rng.choice(durations))
        items.append((200 + j, (2, 1, 1), (64, 1, 1), 0, t, t + d))
        t += d + 10
    rec = make_records(items)
    off = np.array([0, hp_n, hp_n + L], dtype=np.uint64)
    return rec, off


def brute_force_schedule(E, G, D, margin, min_gap):
    """Component-wise earliest feasible first-in-first-out assignment, by full enumeration."""
    H, L = len(E), len(D)
    n_gaps = max(H - 1, 0)
    TAIL = n_gaps  # "after the high-priority trace"
    budget = [(G[i] - margin) if (G[i] >= min_gap and G[i] >= margin) else None for i in range(n_gaps)]
    feasible = []
    for a in itertools.combinations_with_replacement(range(n_gaps + 1), L):  # non-decreasing tuples
        load = [0] * n_gaps
        cnt = [0] * n_gaps
        ok = True
        for j, g in enumerate(a):
            if g == TAIL:
                continue
            if budget[g] is None:
                ok = False
                break
            load[g] += D[j]
            cnt[g] += 1
        if ok and all(budget[g] is None or load[g] <= budget[g] for g in range(n_gaps)):
            feasible.append(a)
    assert feasible  # everything in the tail is always feasible
    best = tuple(min(a[j] for a in feasible) for j in range(L))
    assert best in feasible
    # the earliest schedule also places the most kernels within every prefix of gaps
    for g in range(n_gaps + 1):
        most = max(sum(1 for x in a if x < g) for a in feasible)
        assert sum(1 for x in best if x < g) == most
    fill = [sum(1 for x in best if x == g) for g in range(n_gaps)]
    filled = [sum(D[j] for j, x in enumerate(best) if x == g) for g in range(n_gaps)]
    placed = sum(fill)
    # timeline: HP kernel i ends (gap i opens) at sum(E[:i+1]) + sum(G[:i])
    opens = [sum(E[:i + 1]) + sum(G[:i]) for i in range(H)]
    if L == 0:
        completion = 0
    elif placed == L:
        last = best[-1]
        completion = opens[last] + filled[last]
    else:
        t_end = opens[-1] if H else 0
        completion = t_end + sum(D[placed:])
    return best, fill, filled, placed, completion


@pytest.mark.parametrize("seed", range(40))
def test_p4_bruteforce_tiny(seed):
    rng = np.random.default_rng(1000 + seed)
    H = int(rng.integers(1, 7))
    L = int(rng.integers(0, 7))
    margin = int(rng.choice([0, 500]))
    min_gap = int(rng.choice([0, 2500]))
    durations = [0, 500, 1000, 1500, 2000, 4000]
    gaps = [0, 400, 500, 1500, 2500, 3000, 5000, 9000]
    rec, off = tiny_scenario(rng, H, L, durations, gaps)
    ids, rows, tro = oracle.profile(rec, off)
    E = [int(rec["end_ns"][i] - rec["start_ns"][i]) for i in range(H)]
    G = [int(rec["start_ns"][i + 1] - rec["end_ns"][i]) for i in range(H - 1)]
    D = [int(rec["end_ns"][H + j] - rec["start_ns"][H + j]) for j in range(L)]
    hp = np.array([0], dtype=np.uint32)
    lp = np.array([1], dtype=np.uint32)
    go = traces.gap_offsets(off, hp)
    fc, fn, comp, placed, assign, _ = oracle.gapfill(ids, off, rows, tro, hp, lp, margin, min_gap, go,
                                                     want_assign=True)
    best, fill, filled, n_placed, completion = brute_force_schedule(E, G, D, margin, min_gap)
    tail = max(H - 1, 0)
    got = tuple(tail if x == 0xffffffff else int(x) for x in assign)
    assert got == best
    assert list(fc) == fill
    assert list(fn) == filled
    assert int(placed[0]) == n_placed
    assert int(comp[0]) == completion


# ---------------------------------------------------------------- P5
def numpy_stats(v):
    v = np.sort(np.asarray(v, dtype=np.int64))
    n = v.shape[0]
    if n == 0:
        return [0, 0, 0, 0, 0, 0]
    r50 = -(-50 * n // 100)
    r95 = -(-95 * n // 100)
    return [n, int(v.astype(object).sum()) & U64, int(v[0]), int(v[-1]), int(v[r50 - 1]), int(v[r95 - 1])]


def test_p5_nearest_rank_textbook_examples():
    # worked examples of the nearest-rank definition: ordered list 15 20 35 40 50 -> the 50th
    # percentile is the 3rd value; 3 6 7 8 8 10 13 15 16 20 -> the 50th percentile is the 5th value
    for values, p50, p95 in [([15, 20, 35, 40, 50], 35, 50),
                             ([3, 6, 7, 8, 8, 10, 13, 15, 16, 20], 8, 20),
                             ([7], 7, 7), ([9, 1], 1, 9),
                             (list(range(1, 101)), 50, 95), (list(range(1, 102)), 51, 96)]:
        rng = np.random.default_rng(len(values))
        order = rng.permutation(len(values))
        t = 0
        items = []
        for k in order:
            items.append((3, (1, 1, 1), (1, 1, 1), 0, t, t + values[k]))
            t += values[k] + 5
        _, rows, _ = oracle.profile(make_records(items), np.array([0, len(items)], dtype=np.uint64))
        assert len(rows) == 1
        assert int(rows[0]["exec"]["p50"]) == p50 and int(rows[0]["exec"]["p95"]) == p95
        assert int(rows[0]["exec"]["min"]) == min(values) and int(rows[0]["exec"]["max"]) == max(values)


def test_p5_all_identical_and_all_distinct():
    n = 257
    same = make_records([(4, (2, 2, 2), (8, 8, 1), 64, 1000 * i, 1000 * i + 300) for i in range(n)])
    _, rows, tro = oracle.profile(same, np.array([0, n], dtype=np.uint64))
    assert len(rows) == 1 and list(tro) == [0, 1]
    assert stats_tuple(rows[0]["exec"]) == [n, 300 * n, 300, 300, 300, 300]
    assert stats_tuple(rows[0]["gap"]) == [n - 1, 700 * (n - 1), 700, 700, 700, 700]
    distinct = make_records([(i, (1, 1, 1), (1, 1, 1), 0, 10 * i, 10 * i + 1 + i % 7) for i in range(n)])
    ids, rows, _ = oracle.profile(distinct, np.array([0, n], dtype=np.uint64))
    assert len(rows) == n and np.all(rows["exec"]["count"] == 1)
    assert np.array_equal(rows["kernel_id"], np.sort(ids))
    assert int(rows["gap"]["count"].sum()) == n - 1


@pytest.mark.parametrize("cfg", small_configs(), ids=lambda c: c.name)
def test_p5_groupby_and_order_statistics_match_numpy(cfg):
    rec, off = traces.build(cfg)
    ids, rows, tro = oracle.profile(rec, off)
    ex = rec["end_ns"] - rec["start_ns"]
    for t in range(cfg.n_tasks):
        lo, hi = int(off[t]), int(off[t + 1])
        uid, inv, cnt = np.unique(ids[lo:hi], return_inverse=True, return_counts=True)
        r = rows[int(tro[t]):int(tro[t + 1])]
        assert np.array_equal(r["kernel_id"], uid)
        assert np.array_equal(r["exec"]["count"], cnt.astype(np.uint64))
        gap = np.maximum(0, rec["start_ns"][lo + 1:hi] - rec["end_ns"][lo:hi - 1])
        pick = np.random.default_rng(t).choice(len(uid), size=min(len(uid), 12), replace=False)
        for k in pick:
            assert stats_tuple(r[k]["exec"]) == numpy_stats(ex[lo:hi][inv == k])
            assert stats_tuple(r[k]["gap"]) == numpy_stats(gap[inv[:-1] == k])


def test_p5_sum_wraps_modulo_2_64():
    big = (1 << 62) + 12345
    items = []
    t = -(1 << 62)
    for i in range(5):
        items.append((1, (1, 1, 1), (1, 1, 1), 0, t, t + big))
        t = t + big  # back to back; start of next equals end
        t -= big     # rewind so that timestamps stay inside int64 (overlap -> gap clamps to 0)
    _, rows, _ = oracle.profile(make_records(items), np.array([0, 5], dtype=np.uint64))
    assert int(rows[0]["exec"]["sum"]) == (5 * big) & U64
    assert int(rows[0]["exec"]["p50"]) == big


def test_p5_gapfill_equal_durations_closed_form():
    d = 700
    rng = np.random.default_rng(5)
    H, L = 40, 90
    items = []
    t = 0
    gaps = rng.integers(0, 6000, H)
    for i in range(H):
        items.append((100 + i, (1, 1, 1), (64, 1, 1), 0, t, t + 1000))
        t += 1000 + int(gaps[i])
    t = 0
    for j in range(L):
        items.append((7, (1, 1, 1), (32, 1, 1), 0, t, t + d))
        t += d
    rec = make_records(items)
    off = np.array([0, H, H + L], dtype=np.uint64)
    ids, rows, tro = oracle.profile(rec, off)
    hp = np.array([0], dtype=np.uint32)
    lp = np.array([1], dtype=np.uint32)
    margin, min_gap = 500, 1000
    fc, fn, comp, placed = oracle.gapfill(ids, off, rows, tro, hp, lp, margin, min_gap,
                                          traces.gap_offsets(off, hp))
    remaining = L
    for i in range(H - 1):
        g = int(gaps[i])
        exp = 0 if (g < min_gap or g < margin) else min((g - margin) // d, remaining)
        remaining -= exp
        assert int(fc[i]) == exp and int(fn[i]) == exp * d
    assert int(placed[0]) == L - remaining


# ---------------------------------------------------------------- error statuses
@pytest.mark.parametrize("cfg", small_configs(), ids=lambda c: c.name)
def test_p3_mean_predictor_is_the_median_predictor_on_rows_that_carry_the_mean(cfg):
    """Predicting with SK_j / SG_j (sum // count) must give what the median predictor gives once the rows'
    p50 fields are overwritten with those means: the two only differ in where the prediction is read."""
    rec, off = traces.build(cfg)
    ids, rows, tro = oracle.profile(rec, off)
    _, gap = oracle.measure(rec, off)
    hp, lp = traces.scenarios(cfg)
    if hp.size == 0:
        return
    go = traces.gap_offsets(off, hp)
    swapped = rows.copy()
    for blk in ("exec", "gap"):
        cnt = rows[blk]["count"].astype(np.uint64)
        swapped[blk]["p50"] = np.where(cnt > 0, rows[blk]["sum"] // np.maximum(cnt, 1), 0).astype(np.int64)
    a = oracle.gapfill(ids, off, rows, tro, hp, lp, cfg.margin_ns, 0, go, predictor=1)
    b = oracle.gapfill(ids, off, swapped, tro, hp, lp, cfg.margin_ns, 0, go, predictor=0)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    assert not all(np.array_equal(x, y) for x, y in zip(a, oracle.gapfill(ids, off, rows, tro, hp, lp, cfg.margin_ns, 0, go)))
    for fb in (False, True):
        a = oracle.replay(ids, off, rows, tro, gap, hp, lp, cfg.margin_ns, 0, fb, go, predictor=1)
        b = oracle.replay(ids, off, swapped, tro, gap, hp, lp, cfg.margin_ns, 0, fb, go, predictor=0)
        assert all(np.array_equal(x, y) for x, y in zip(a, b))
    with pytest.raises(oracle.OracleError) as e:
        oracle.gapfill(ids, off, rows, tro, hp, lp, 0, 0, go, predictor=2)
    assert e.value.status == oracle.INVALID_ARG


# ---------------------------------------------------------------- P6
def test_p6_measure_is_end_minus_start_and_next_start_minus_end():
    rec = make_records([(1, (1, 1, 1), (64, 1, 1), 0, 10, 25), (2, (1, 1, 1), (64, 1, 1), 0, 30, 31),
                        (1, (1, 1, 1), (64, 1, 1), 0, 29, 40),       # starts before the previous one ends
                        (3, (1, 1, 1), (64, 1, 1), 0, 100, 100), (3, (1, 1, 1), (64, 1, 1), 0, 107, 110)])
    off = np.array([0, 3, 3, 5], dtype=np.uint64)
    ex, gp = oracle.measure(rec, off)
    assert ex.tolist() == [15, 1, 11, 0, 3]
    assert gp.tolist() == [5, 0, -1, 7, -1]
    cfg = traces.config(0)
    rec, off = traces.build(cfg)
    ex, gp = oracle.measure(rec, off)
    assert np.array_equal(ex, rec["end_ns"] - rec["start_ns"])
    nxt = np.roll(rec["start_ns"], -1) - rec["end_ns"]
    last = np.zeros(rec.shape[0], dtype=bool)
    last[(off[1:][off[1:] > off[:-1]] - 1).astype(np.int64)] = True
    assert np.array_equal(gp, np.where(last, -1, np.maximum(nxt, 0)))


def replay_inputs(golden):
    hp_ids, lp_ids = golden["hp_ids"], golden["lp_ids"]
    ids = np.array(hp_ids + lp_ids, dtype=np.uint64)
    off = np.array([0, len(hp_ids), len(ids)], dtype=np.uint64)
    rows = np.zeros(len(golden["rows"]), dtype=oracle.ROW_DTYPE)
    for k, r in enumerate(golden["rows"]):
        rows[k]["kernel_id"] = r["kernel_id"]
        rows[k]["task"] = r["task"]
        rows[k]["exec"]["p50"] = r["exec_p50"]
        rows[k]["gap"]["p50"] = r["gap_p50"]
    tro = np.array([0, 2, 3], dtype=np.uint64)
    return ids, off, rows, tro


def test_p6_replay_hand_worked(golden_dir):
    with open(os.path.join(golden_dir, "p6_replay_hand_worked.json")) as f:
        golden = json.load(f)
    ids, off, rows, tro = replay_inputs(golden)
    hp, lp = np.array([0], dtype=np.uint32), np.array([1], dtype=np.uint32)
    go = traces.gap_offsets(off, hp)
    for case in golden["cases"]:
        actual = np.array(case["actual_gap_ns"] + [-1] + [1] * (len(golden["lp_ids"]) - 1) + [-1], dtype=np.int64)
        for feedback, key in ((False, "no_feedback"), (True, "feedback")):
            fc, fn, delay, placed = oracle.replay(ids, off, rows, tro, actual, hp, lp, case["margin_ns"],
                                                  case["min_gap_ns"], feedback, go)
            exp = case[key]
            assert fc.tolist() == exp["fill_count"], (case, key)
            assert fn.tolist() == exp["filled_ns"], (case, key)
            assert int(delay[0]) == exp["hp_delay_ns"], (case, key)
            assert int(placed[0]) == exp["lp_placed"], (case, key)


def replay_by_prefix_sums(E_pred_gap, actual, D, margin, min_gap, feedback):
    """The replay of one scenario written with prefix sums and searches instead of a kernel-by-kernel loop."""
    ps = np.concatenate([[0], np.cumsum(np.asarray(D, dtype=np.int64))])
    p, delay, fills, filled = 0, 0, [], []
    for G, A in zip(E_pred_gap, actual):
        c = 0
        if G >= min_gap and G >= margin:
            # kernels p .. p+c-1 fit the predicted budget: largest c with ps[p+c] - ps[p] <= G - margin
            c = int(np.searchsorted(ps, ps[p] + (G - margin), side="right")) - 1 - p
            if feedback:
                # kernel p+k is issued only if the time filled before it, ps[p+k] - ps[p], is below the actual gap
                started = int(np.searchsorted(ps[p:p + c] - ps[p], A, side="left"))
                c = min(c, started)
        f = int(ps[p + c] - ps[p])
        fills.append(c)
        filled.append(f)
        delay += max(0, f - A)
        p += c
    return fills, filled, delay, p


@pytest.mark.parametrize("cfg", small_configs(), ids=lambda c: c.name)
def test_p6_replay_ties(cfg):
    rec, off = traces.build(cfg)
    ids, rows, tro = oracle.profile(rec, off)
    _, gap = oracle.measure(rec, off)
    hp, lp = traces.scenarios(cfg)
    if hp.size == 0:
        return
    go = traces.gap_offsets(off, hp)
    for margin, min_gap in ((cfg.margin_ns, 0), (0, 20000)):
        ref = oracle.gapfill(ids, off, rows, tro, hp, lp, margin, min_gap, go)
        # without feedback the decisions are those of the gap fill; the delay is what runs past the actual gap
        fc, fn, delay, placed = oracle.replay(ids, off, rows, tro, gap, hp, lp, margin, min_gap, False, go)
        assert np.array_equal(fc, ref[0]) and np.array_equal(fn, ref[1]) and np.array_equal(placed, ref[3])
        for s in range(hp.size):
            h0 = int(off[hp[s]])
            n_g = int(go[s + 1] - go[s])
            a = gap[h0:h0 + n_g]
            assert int(delay[s]) == int(np.maximum(fn[int(go[s]):int(go[s + 1])] - a, 0).sum())
        # gaps that never end early: feedback changes nothing and nothing is delayed
        huge = np.where(gap < 0, -1, np.int64(1) << 60)
        for fb in (False, True):
            fc2, fn2, delay2, placed2 = oracle.replay(ids, off, rows, tro, huge, hp, lp, margin, min_gap, fb, go)
            assert np.array_equal(fc2, ref[0]) and np.array_equal(fn2, ref[1]) and not delay2.any()
        # gaps that end at once: with feedback nothing is issued
        zero = np.where(gap < 0, -1, 0)
        fc3, fn3, delay3, placed3 = oracle.replay(ids, off, rows, tro, zero, hp, lp, margin, min_gap, True, go)
        assert not fc3.any() and not fn3.any() and not delay3.any() and not placed3.any()
        # with feedback, a gap's overrun is shorter than the last kernel issued into it, and the closed form agrees
        fc4, fn4, delay4, placed4 = oracle.replay(ids, off, rows, tro, gap, hp, lp, margin, min_gap, True, go)
        for s in range(min(hp.size, 8)):
            h0, l0, l1 = int(off[hp[s]]), int(off[lp[s]]), int(off[lp[s] + 1])
            n_g = int(go[s + 1] - go[s])
            lut_e = {int(r["kernel_id"]): int(r["exec"]["p50"]) for r in rows[int(tro[lp[s]]):int(tro[lp[s] + 1])]}
            lut_g = {int(r["kernel_id"]): int(r["gap"]["p50"]) for r in rows[int(tro[hp[s]]):int(tro[hp[s] + 1])]}
            D = [lut_e[int(i)] for i in ids[l0:l1]]
            Gp = [lut_g[int(i)] for i in ids[h0:h0 + n_g]]
            for fb, got in ((False, (fc, fn, delay, placed)), (True, (fc4, fn4, delay4, placed4))):
                fills, filled, dl, p = replay_by_prefix_sums(Gp, gap[h0:h0 + n_g].tolist(), D, margin, min_gap, fb)
                sl = slice(int(go[s]), int(go[s + 1]))
                assert got[0][sl].tolist() == fills and got[1][sl].tolist() == filled
                assert int(got[2][s]) == dl and int(got[3][s]) == p
            p = 0
            for g in range(n_g):
                c = int(fc4[int(go[s]) + g])
                if c:
                    assert int(fn4[int(go[s]) + g]) - D[p + c - 1] < int(gap[h0 + g])
                p += c


# ---------------------------------------------------------------- P7
def prio_inputs(hp_launches, hp_gap, lp):
    """Rows and IDs for one high-priority task (one kernel, predicted idle time hp_gap) and the given low-priority
    tasks (one kernel ID per distinct duration of a task)."""
    ids, off, rows, tro = [1] * hp_launches, [0, hp_launches], [], [0]
    rows.append((1, 0, 7, hp_gap))
    tro.append(1)
    for t, task in enumerate(lp, start=1):
        durs = sorted(set(task["durations"]))
        for d in durs:
            rows.append((1000 * t + durs.index(d), t, d, 1))
        ids += [1000 * t + durs.index(d) for d in task["durations"]]
        off.append(len(ids))
        tro.append(len(rows))
    r = np.zeros(len(rows), dtype=oracle.ROW_DTYPE)
    for k, (kid, task, e, g) in enumerate(rows):
        r[k]["kernel_id"], r[k]["task"] = kid, task
        r[k]["exec"]["p50"], r[k]["gap"]["p50"] = e, g
    lp_task = np.arange(1, len(lp) + 1, dtype=np.uint32)
    lp_prio = np.array([task["prio"] for task in lp], dtype=np.uint32)
    return (np.array(ids, dtype=np.uint64), np.array(off, dtype=np.uint64), r, np.array(tro, dtype=np.uint64),
            np.array([0], dtype=np.uint32), np.array([0, len(lp)], dtype=np.uint64), lp_task, lp_prio)


@pytest.mark.parametrize("case", ["abc", "equal_priority", "longest_fit"])
def test_p7_prio_fill_hand_worked(golden_dir, case):
    with open(os.path.join(golden_dir, "p7_prio_fill_hand_worked.json")) as f:
        golden = json.load(f)
    exp = golden["cases"][case]
    ids, off, rows, tro, hp, lo, lt, lq = prio_inputs(golden["hp_launches"], golden["hp_gap"], exp["lp"])
    go = traces.gap_offsets(off, hp)
    fc, fn, placed, placed_ns, issue, ioff = oracle.prio_fill(ids, off, rows, tro, hp, lo, lt, lq, 0, 0, go, want_issue=True)
    assert fc.tolist() == exp["fill_count"] and fn.tolist() == exp["filled_ns"]
    assert placed.tolist() == exp["lp_placed"] and placed_ns.tolist() == exp["lp_placed_ns"]
    assert issue[: int(placed.sum())].tolist() == exp["issue_entry"]


def random_prio_scenarios(cfg, rng, n_scen, max_lp=4):
    hp = rng.integers(0, cfg.n_tasks, n_scen).astype(np.uint32)
    k = rng.integers(0, max_lp + 1, n_scen)
    lo = np.zeros(n_scen + 1, dtype=np.uint64)
    np.cumsum(k, out=lo[1:])
    lt = rng.integers(0, cfg.n_tasks, int(lo[-1])).astype(np.uint32)
    lq = rng.integers(1, 10, int(lo[-1])).astype(np.uint32)
    lq[rng.random(lq.shape[0]) < 0.5] = 4      # plenty of equal priorities
    return hp, lo, lt, lq


@pytest.mark.parametrize("cfg", small_configs(), ids=lambda c: c.name)
def test_p7_prio_fill_ties_and_rule(cfg):
    rec, off = traces.build(cfg)
    ids, rows, tro = oracle.profile(rec, off)
    rng = np.random.default_rng(77)
    # one low-priority task: the gap fill itself, whatever the level
    hp, lp = traces.scenarios(cfg)
    if hp.size:
        go = traces.gap_offsets(off, hp)
        ref = oracle.gapfill(ids, off, rows, tro, hp, lp, cfg.margin_ns, 0, go)
        lo = np.arange(hp.size + 1, dtype=np.uint64)
        got = oracle.prio_fill(ids, off, rows, tro, hp, lo, lp, rng.integers(1, 10, hp.size).astype(np.uint32),
                               cfg.margin_ns, 0, go)
        assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1]) and np.array_equal(got[2], ref[3])
    # several: replay the issue log and check every decision against the rule written as a sort key
    hp, lo, lt, lq = random_prio_scenarios(cfg, rng, 12)
    go = traces.gap_offsets(off, hp)
    margin, min_gap = cfg.margin_ns, 3000
    fc, fn, placed, placed_ns, issue, ioff = oracle.prio_fill(ids, off, rows, tro, hp, lo, lt, lq, margin, min_gap, go,
                                                             want_issue=True)
    for s in range(hp.size):
        e0, K = int(lo[s]), int(lo[s + 1] - lo[s])
        h0, H = int(off[hp[s]]), int(off[hp[s] + 1] - off[hp[s]])
        lut_g = {int(r["kernel_id"]): int(r["gap"]["p50"]) for r in rows[int(tro[hp[s]]):int(tro[hp[s] + 1])]}
        D = []
        for k in range(K):
            t = int(lt[e0 + k])
            lut_e = {int(r["kernel_id"]): int(r["exec"]["p50"]) for r in rows[int(tro[t]):int(tro[t + 1])]}
            D.append([lut_e[int(i)] for i in ids[int(off[t]):int(off[t + 1])]])
        nxt, stamp, clock, at = [0] * K, list(range(K)), K, int(ioff[s])
        count = [0] * K
        for g in range(max(H - 1, 0)):
            G = lut_g[int(ids[h0 + g])]
            c = f = 0
            if G >= min_gap and G >= margin:
                r = G - margin
                while True:
                    cand = sorted((int(lq[e0 + k]), -D[k][nxt[k]], stamp[k], k) for k in range(K)
                                  if nxt[k] < len(D[k]) and D[k][nxt[k]] <= r)
                    if not cand:
                        break
                    k = cand[0][3]
                    assert int(issue[at]) == k, (s, g)
                    at += 1
                    r -= D[k][nxt[k]]
                    f += D[k][nxt[k]]
                    c += 1
                    nxt[k] += 1
                    count[k] += 1
                    stamp[k] = clock
                    clock += 1
            assert int(fc[int(go[s]) + g]) == c and int(fn[int(go[s]) + g]) == f, (s, g)
        assert [int(x) for x in placed[e0:e0 + K]] == count
        assert at - int(ioff[s]) == sum(count)
    # argument errors
    for bad_prio in (0, 10):
        with pytest.raises(oracle.OracleError) as e:
            oracle.prio_fill(ids, off, rows, tro, hp[:1], np.array([0, 1], dtype=np.uint64), np.array([0], dtype=np.uint32),
                             np.array([bad_prio], dtype=np.uint32), 0, 0, traces.gap_offsets(off, hp[:1]))
        assert e.value.status == oracle.INVALID_ARG


# ---------------------------------------------------------------- P8
NO_SCENARIO, NO_TASK = np.uint64(2**64 - 1), np.uint32(2**32 - 1)


def pairing_golden(golden):
    sc = golden["scenarios"]
    hp = np.array([x["hp"] for x in sc], dtype=np.uint32)
    lp = np.array([x["lp"] for x in sc], dtype=np.uint32)
    go = np.zeros(len(sc) + 1, dtype=np.uint64)
    np.cumsum([len(x["filled_ns"]) for x in sc], out=go[1:])
    fn = np.array([v for x in sc for v in x["filled_ns"]], dtype=np.int64)
    comp = np.array([x["lp_completion_ns"] for x in sc], dtype=np.int64)
    exp = (np.array(golden["scenario_filled_ns"], dtype=np.int64),
           np.array([NO_SCENARIO if v < 0 else v for v in golden["best_scenario"]], dtype=np.uint64),
           np.array([NO_TASK if v < 0 else v for v in golden["best_lp"]], dtype=np.uint32),
           np.array(golden["best_filled_ns"], dtype=np.int64))
    return hp, lp, golden["n_tasks"], go, fn, comp, exp


def test_p8_pairing_hand_worked(golden_dir):
    with open(os.path.join(golden_dir, "p8_pairing_hand_worked.json")) as f:
        golden = json.load(f)
    hp, lp, n_tasks, go, fn, comp, exp = pairing_golden(golden)
    got = oracle.pairing_best(hp, lp, n_tasks, go, fn, comp)
    for a, b in zip(got, exp):
        assert np.array_equal(a, b)


def pairing_by_lexsort(hp, lp, n_tasks, go, fn, comp):
    total = np.array([fn[int(go[s]):int(go[s + 1])].sum() for s in range(hp.size)], dtype=np.int64)
    best_s = np.full(n_tasks, NO_SCENARIO, dtype=np.uint64)
    best_lp = np.full(n_tasks, NO_TASK, dtype=np.uint32)
    best_f = np.zeros(n_tasks, dtype=np.int64)
    order = np.lexsort((np.arange(hp.size), comp, -total, hp))      # last key first: task, most filled, earliest done, first
    first = np.ones(hp.size, dtype=bool)
    first[1:] = hp[order][1:] != hp[order][:-1]
    for s in order[first]:
        best_s[hp[s]], best_lp[hp[s]], best_f[hp[s]] = s, lp[s], total[s]
    return total, best_s, best_lp, best_f


def random_pairing(rng, n_tasks, n_scen, max_gaps, values):
    hp = rng.integers(0, n_tasks, n_scen).astype(np.uint32)
    lp = rng.integers(0, n_tasks, n_scen).astype(np.uint32)
    go = np.zeros(n_scen + 1, dtype=np.uint64)
    np.cumsum(rng.integers(0, max_gaps + 1, n_scen), out=go[1:])
    fn = rng.integers(0, values, int(go[-1])).astype(np.int64)
    comp = rng.integers(0, 4, n_scen).astype(np.int64)            # many ties
    return hp, lp, go, fn, comp


def test_p8_pairing_against_lexsort():
    rng = np.random.default_rng(8)
    for n_tasks, n_scen, max_gaps, values in ((1, 1, 0, 1), (7, 200, 3, 2), (50, 40, 9, 1000), (9, 3000, 2, 3), (300, 5000, 40, 10**12)):
        hp, lp, go, fn, comp = random_pairing(rng, n_tasks, n_scen, max_gaps, values)
        got = oracle.pairing_best(hp, lp, n_tasks, go, fn, comp)
        for a, b in zip(got, pairing_by_lexsort(hp, lp, n_tasks, go, fn, comp)):
            assert np.array_equal(a, b)
    got = oracle.pairing_best(np.zeros(0, np.uint32), np.zeros(0, np.uint32), 3, np.zeros(1, np.uint64), np.zeros(0, np.int64),
                              np.zeros(0, np.int64))
    assert got[0].size == 0 and (got[1] == NO_SCENARIO).all() and (got[2] == NO_TASK).all() and (got[3] == 0).all()
    with pytest.raises(oracle.OracleError):
        oracle.pairing_best(np.array([3], np.uint32), np.array([0], np.uint32), 3, np.zeros(2, np.uint64), np.zeros(0, np.int64),
                            np.zeros(1, np.int64))


def test_p8_pairing_of_a_grid_of_gap_fills():
    cfg = traces.config(1, n_tasks=8, launches=3000)          # 4 x 4 combinations
    rec, off = traces.build(cfg)
    ids, rows, tro = oracle.profile(rec, off)
    hp, lp = traces.scenarios(cfg)
    assert hp.size == 16
    go = traces.gap_offsets(off, hp)
    fc, fn, comp, placed = oracle.gapfill(ids, off, rows, tro, hp, lp, cfg.margin_ns, cfg.min_gap_ns, go)
    total, best_s, best_lp, best_f = oracle.pairing_best(hp, lp, cfg.n_tasks, go, fn, comp)
    for t in range(cfg.n_tasks):
        mine = [s for s in range(hp.size) if hp[s] == t]
        if not mine:
            assert best_s[t] == NO_SCENARIO and best_lp[t] == NO_TASK and best_f[t] == 0
            continue
        sums = {s: sum(int(v) for v in fn[int(go[s]):int(go[s + 1])]) for s in mine}
        top = max(sums.values())
        cands = [s for s in mine if sums[s] == top]
        soonest = min(int(comp[s]) for s in cands)
        pick = min(s for s in cands if int(comp[s]) == soonest)
        assert int(best_s[t]) == pick and int(best_lp[t]) == int(lp[pick]) and int(best_f[t]) == top
        assert all(int(total[s]) == sums[s] for s in mine)


# ---------------------------------------------------------------- P9
STAT_FIELDS = ("count", "sum", "min", "max", "p50", "p95")


def rows_from_json(items):
    rows = np.zeros(len(items), dtype=oracle.ROW_DTYPE)
    for r, it in zip(rows, items):
        r["kernel_id"], r["task"] = it["id"], it["task"]
        for blk in ("exec", "gap"):
            for f, v in zip(STAT_FIELDS, it[blk]):
                r[blk][f] = v
    return rows


def offsets_of(rows, n_tasks):
    off = np.zeros(n_tasks + 1, dtype=np.uint64)
    np.cumsum(np.bincount(rows["task"].astype(np.int64), minlength=n_tasks), out=off[1:])
    return off


def test_p9_merge_hand_worked(golden_dir):
    with open(os.path.join(golden_dir, "p9_merge_hand_worked.json")) as f:
        golden = json.load(f)
    n_tasks = golden["n_tasks"]
    a, b, exp = rows_from_json(golden["a"]), rows_from_json(golden["b"]), rows_from_json(golden["merged"])
    got, off = oracle.profile_merge(a, offsets_of(a, n_tasks), b, offsets_of(b, n_tasks))
    assert got.tobytes() == exp.tobytes()
    assert np.array_equal(off, offsets_of(exp, n_tasks))


def split_runs(rec, off, cut):
    """Every task's trace cut at fraction `cut` into two runs: (records, offsets) of the first and of the second."""
    first, second, o1, o2 = [], [], [0], [0]
    for t in range(off.size - 1):
        a, b = int(off[t]), int(off[t + 1])
        c = a + int((b - a) * cut)
        first.append(rec[a:c])
        second.append(rec[c:b])
        o1.append(o1[-1] + c - a)
        o2.append(o2[-1] + b - c)
    return (np.concatenate(first), np.array(o1, dtype=np.uint64)), (np.concatenate(second), np.array(o2, dtype=np.uint64))


@pytest.mark.parametrize("cfg", small_configs(), ids=lambda c: c.name)
def test_p9_merge_of_runs_is_the_profile_without_the_idle_time_between_runs(cfg):
    rec, off = traces.build(cfg)
    (r1, o1), (r2, o2) = split_runs(rec, off, 0.37)
    _, rows1, tro1 = oracle.profile(r1, o1)
    _, rows2, tro2 = oracle.profile(r2, o2)
    merged, mtro = oracle.profile_merge(rows1, tro1, rows2, tro2)
    ids, whole, wtro = oracle.profile(rec, off)
    # same IDs in the same order, same execution-time statistics but for the percentiles
    assert np.array_equal(mtro, wtro)
    assert np.array_equal(merged["kernel_id"], whole["kernel_id"]) and np.array_equal(merged["task"], whole["task"])
    for f in ("count", "sum", "min", "max"):
        assert np.array_equal(merged["exec"][f], whole["exec"][f]), f
    # idle times: those of the whole trace except the one that follows the last launch of a task's first run
    ex, gp = oracle.measure(rec, off)
    gp = gp.copy()
    for t in range(off.size - 1):
        if o1[t + 1] > o1[t] and o2[t + 1] > o2[t]:
            gp[int(off[t]) + int(o1[t + 1] - o1[t]) - 1] = -1
    for t in range(off.size - 1):
        a, b = int(off[t]), int(off[t + 1])
        for r in range(int(mtro[t]), int(mtro[t + 1])):
            g = gp[a:b][(ids[a:b] == merged["kernel_id"][r]) & (gp[a:b] >= 0)]
            row = merged["gap"][r]
            assert int(row["count"]) == g.size
            if g.size:
                assert int(row["sum"]) == int(g.sum()) and int(row["min"]) == int(g.min()) and int(row["max"]) == int(g.max())
                assert int(row["min"]) <= int(row["p50"]) <= int(row["p95"]) <= int(row["max"])
            else:
                assert all(int(row[f]) == 0 for f in STAT_FIELDS)
    # identity and symmetry
    empty = np.zeros(0, dtype=oracle.ROW_DTYPE)
    zero = np.zeros(off.size, dtype=np.uint64)
    same, same_off = oracle.profile_merge(rows1, tro1, empty, zero)
    assert same.tobytes() == rows1.tobytes() and np.array_equal(same_off, tro1)
    same, _ = oracle.profile_merge(empty, zero, rows1, tro1)
    assert same.tobytes() == rows1.tobytes()
    other, other_off = oracle.profile_merge(rows2, tro2, rows1, tro1)
    assert np.array_equal(other_off, mtro)
    for blk in ("exec", "gap"):
        for f in ("count", "sum", "min", "max"):
            assert np.array_equal(other[blk][f], merged[blk][f])
        # the percentiles are those of the input with more samples
        for r in range(merged.shape[0]):
            t, kid = int(merged["task"][r]), merged["kernel_id"][r]
            src = [x for x in (rows1[int(tro1[t]):int(tro1[t + 1])], rows2[int(tro2[t]):int(tro2[t + 1])])]
            cands = [x[x["kernel_id"] == kid] for x in src]
            cands = [c[0][blk] for c in cands if c.size and int(c[0][blk]["count"]) > 0]
            if cands:
                best = max(cands, key=lambda c: int(c["count"]))      # (max keeps the first of equals)
                assert int(merged[blk]["p50"][r]) == int(best["p50"]) and int(merged[blk]["p95"][r]) == int(best["p95"])
    # capacity and argument errors
    with pytest.raises(oracle.OracleError) as e:
        oracle.profile_merge(rows1, tro1, rows2, tro2, row_capacity=max(merged.shape[0] - 1, 0))
    assert e.value.status == oracle.ROW_CAPACITY and e.value.n_rows == merged.shape[0]
    if rows1.shape[0] > 1:
        bad = rows1.copy()
        bad["task"][0] = 99
        with pytest.raises(oracle.OracleError):
            oracle.profile_merge(bad, tro1, rows2, tro2)


# ---------------------------------------------------------------- P10: several measured runs in one trace
@pytest.mark.parametrize("case", ["two_runs_of_six", "three_runs_of_four", "run_numbers_need_not_be_consecutive_or_ascending"])
def test_p10_runs_hand_worked(p1, golden_dir, case):
    g1, rec, off = p1
    with open(os.path.join(golden_dir, "p10_runs_hand_worked.json")) as f:
        g = json.load(f)["cases"][case]
    hp = rec[:12].copy()
    hp["run"] = g["run_of_launch"]
    _, rows, _ = oracle.profile(hp, np.array([0, 12], dtype=np.uint64))
    assert len(rows) == 3
    for r, name in zip(rows, g1["rows_in_order"][:3]):
        assert stats_tuple(r["exec"]) == g1["rows"][name]["exec"]      # execution times do not depend on the runs
        assert stats_tuple(r["gap"]) == g["gap"][name], name
    if "SG_C" in g:
        c = rows[2]
        assert Fraction(int(c["gap"]["sum"]), int(c["gap"]["count"])) == g["SG_C"]
    _, gp = oracle.measure(hp, np.array([0, 12], dtype=np.uint64))
    ends = [i for i in range(12) if i == 11 or g["run_of_launch"][i + 1] != g["run_of_launch"][i]]
    assert [i for i in range(12) if gp[i] < 0] == ends


@pytest.mark.parametrize("cfg", small_configs(), ids=lambda c: c.name)
@pytest.mark.parametrize("runs", [2, 5])
def test_p10_runs_in_one_trace_against_numpy_and_against_the_merge_of_separate_profiles(cfg, runs):
    cfg = traces.config(cfg.index, runs=runs, **dict(cfg.overrides))
    rec, off = traces.build(cfg)
    assert int(rec["run"].max()) == runs - 1
    ids, rows, tro = oracle.profile(rec, off)
    plain = rec.copy()
    plain["run"] = 0
    ids0, rows0, tro0 = oracle.profile(plain, off)
    # the run number is no part of the identity, and execution times do not depend on it
    assert np.array_equal(ids, ids0) and np.array_equal(tro, tro0)
    assert np.array_equal(rows["kernel_id"], rows0["kernel_id"]) and rows["exec"].tobytes() == rows0["exec"].tobytes()
    n_runs = sum(len(np.unique(rec["run"][int(off[t]):int(off[t + 1])])) for t in range(cfg.n_tasks))
    assert int(rows["gap"]["count"].sum()) == rec.shape[0] - n_runs          # N - 1 idle times per run
    # every field, percentiles included, from plain numpy on the samples that the definition keeps
    for t in range(cfg.n_tasks):
        lo, hi = int(off[t]), int(off[t + 1])
        same_run = rec["run"][lo + 1:hi] == rec["run"][lo:hi - 1]
        gap = np.maximum(0, rec["start_ns"][lo + 1:hi] - rec["end_ns"][lo:hi - 1])
        r = rows[int(tro[t]):int(tro[t + 1])]
        pick = np.random.default_rng(t).choice(len(r), size=min(len(r), 16), replace=False)
        for k in pick:
            mine = ids[lo:hi - 1] == r["kernel_id"][k]
            assert stats_tuple(r[k]["gap"]) == numpy_stats(gap[mine & same_run])
    # the runs profiled one by one and merged: the same counts, sums, minima and maxima
    merged, mtro = None, None
    for q in range(runs):
        keep = rec["run"] == q
        sub = plain[keep]
        sub_off = np.zeros(cfg.n_tasks + 1, dtype=np.uint64)
        np.cumsum([int(keep[int(off[t]):int(off[t + 1])].sum()) for t in range(cfg.n_tasks)], out=sub_off[1:])
        _, rq, tq = oracle.profile(sub, sub_off)
        merged, mtro = (rq, tq) if merged is None else oracle.profile_merge(merged, mtro, rq, tq)
    assert np.array_equal(mtro, tro) and np.array_equal(merged["kernel_id"], rows["kernel_id"])
    for blk in ("exec", "gap"):
        for f in ("count", "sum", "min", "max"):
            assert np.array_equal(merged[blk][f], rows[blk][f]), (blk, f)


def test_oracle_error_statuses():
    rec = make_records([(1, (1, 1, 1), (1, 1, 1), 0, 10, 5)])
    with pytest.raises(oracle.OracleError) as e:
        oracle.profile(rec, np.array([0, 1], dtype=np.uint64))
    assert e.value.status == oracle.BAD_RECORD
    ok = make_records([(1, (1, 1, 1), (1, 1, 1), 0, 0, 5), (2, (1, 1, 1), (1, 1, 1), 0, 6, 9)])
    for bad in ([0, 3], [1, 2], [0, 2, 1, 2]):
        with pytest.raises(oracle.OracleError) as e:
            oracle.profile(ok, np.array(bad, dtype=np.uint64))
        assert e.value.status == oracle.INVALID_ARG
    with pytest.raises(oracle.OracleError) as e:
        oracle.profile(ok, np.array([0, 2], dtype=np.uint64), row_capacity=1)
    assert e.value.status == oracle.ROW_CAPACITY and e.value.n_rows == 2
    ids, rows, tro = oracle.profile(ok, np.array([0, 1, 2], dtype=np.uint64))
    hp = np.array([0], dtype=np.uint32)
    lp = np.array([1], dtype=np.uint32)
    off = np.array([0, 1, 2], dtype=np.uint64)
    wrong = ids.copy()
    wrong[1] ^= np.uint64(1)
    with pytest.raises(oracle.OracleError) as e:
        oracle.gapfill(wrong, off, rows, tro, hp, lp, 0, 0, traces.gap_offsets(off, hp))
    assert e.value.status == oracle.UNKNOWN_ID


def test_empty_inputs():
    rec = np.zeros(0, dtype=traces.LAUNCH_DTYPE)
    ids, rows, tro = oracle.profile(rec, np.array([0, 0, 0], dtype=np.uint64))
    assert len(ids) == 0 and len(rows) == 0 and list(tro) == [0, 0, 0]
    # empty tasks between non-empty ones; scenarios with H <= 1 and L == 0
    one = make_records([(1, (1, 1, 1), (1, 1, 1), 0, 0, 700), (2, (1, 1, 1), (1, 1, 1), 0, 0, 300),
                        (2, (1, 1, 1), (1, 1, 1), 0, 400, 800)])
    off = np.array([0, 0, 1, 1, 3, 3], dtype=np.uint64)
    ids, rows, tro = oracle.profile(one, off)
    assert list(tro) == [0, 0, 1, 1, 2, 2]
    assert stats_tuple(rows[0]["gap"]) == [0, 0, 0, 0, 0, 0]
    hp = np.array([1, 0, 1, 3], dtype=np.uint32)
    lp = np.array([3, 3, 0, 0], dtype=np.uint32)
    go = traces.gap_offsets(off, hp)
    assert list(go) == [0, 0, 0, 0, 1]
    fc, fn, comp, placed = oracle.gapfill(ids, off, rows, tro, hp, lp, 0, 0, go)
    d = int(rows[1]["exec"]["p50"])
    assert d == 300
    assert int(comp[0]) == 700 + 2 * d and int(placed[0]) == 0   # H == 1: no gap, LP runs afterwards
    assert int(comp[1]) == 2 * d                                   # H == 0
    assert int(comp[2]) == 0 and int(placed[2]) == 0               # L == 0
    assert int(comp[3]) == 0 and list(fc) == [0]                   # L == 0 with one (unused) gap
