"""Seeded sweep over all entry points at once: random task shapes, scenario lists, margins, thresholds and
predictors, every output compared with the CPU oracle (needs an MI355X)."""
import numpy as np
import pytest

from paper_2311_10359_amd import traces
from parity_util import check_gapfill, check_profile
from test_gpu_pairing import check_pairing
from test_gpu_parity import mixed_trace
from test_gpu_prio import check_prio, prio_lists
from test_gpu_replay import check_measure, check_replay

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", range(24))
def test_sweep(seed):
    rng = np.random.default_rng(50000 + seed)
    n_tasks = int(rng.integers(2, 14))
    max_len = int(rng.choice([300, 4097, 8193, 20000, 40000]))
    wide = bool(rng.random() < 0.2)
    rec, off, lens = mixed_trace(7000 + seed, n_tasks, max_len, wide=wide)
    print(f"seed {seed}: lengths {lens}, values beyond 32 bits: {wide}", flush=True)
    prof, d_off, o_prof = check_profile(rec, off)
    n_scen = int(rng.integers(1, 60))
    hp = rng.integers(0, n_tasks, n_scen).astype(np.uint32)
    lp = rng.integers(0, n_tasks, n_scen).astype(np.uint32)
    margin = int(rng.choice([0, 1, 500, 10**5]))
    min_gap = int(rng.choice([0, 7, 10**4]))
    predictor = int(rng.integers(0, 2))
    got = check_gapfill(prof, d_off, off, o_prof, hp, lp, margin, min_gap, predictor=predictor)
    go = traces.gap_offsets(off, hp)
    check_pairing(hp, lp, n_tasks, go, got.filled_ns.cpu().numpy(), got.lp_completion_ns.cpu().numpy())
    # (with values beyond 32 bits the 64-bit kernels take the replay and the priority queues)
    d_gap, gap = check_measure(rec, off)
    check_replay(prof, d_off, off, o_prof, d_gap, gap, hp, lp, margin, min_gap, predictor=predictor)
    k_max = int(rng.choice([1, 2, 3, 4, 6, 9, 20, 70]))
    hp2, lo, lt, lq = prio_lists(rng, n_tasks, int(rng.integers(1, 80)), k_max)
    check_prio(prof, d_off, off, o_prof, hp2, lo, lt, lq, margin, min_gap, predictor=predictor)
