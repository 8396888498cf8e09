// Gap filling with several low-priority tasks per scenario: Algorithm 1 calling the whole of
// Algorithm 2 (BestPrioFit) over the priority queues Q1..Q9.
#pragma once

#include "common.hip.h"
#include "gapfill_kernels.hip.h"

namespace fikit {

constexpr uint32_t PF_MAX_LP = FIKIT_PRIO_MAX_LP;   // low-priority tasks of one scenario (one lane each, one wave at most)

// Checks the scenario arguments, records in role[t] how each task is used and leaves the largest
// number of low-priority tasks of a scenario in ctrl->n_class[3].
__global__ void k_pf_scenarios(const uint64_t* __restrict__ off, uint32_t n_tasks, const uint32_t* __restrict__ hp_task,
                               const uint64_t* __restrict__ lp_off, const uint32_t* __restrict__ lp_task,
                               const uint32_t* __restrict__ lp_prio, uint64_t n_scen, uint64_t n_entries,
                               const uint64_t* __restrict__ gap_off, uint32_t* __restrict__ role, Ctrl* ctrl) {
  if (ctrl->status & ERR_OFFSETS) return;
  const uint64_t s = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  uint32_t k_here = 0;
  if (s < n_scen) {
    const uint32_t hp = hp_task[s];
    const uint64_t e0 = lp_off[s], e1 = lp_off[s + 1];
    if (hp >= n_tasks) {
      atomicOr(&ctrl->status, ERR_TASK_INDEX);
    } else if (e1 < e0 || e1 > n_entries || (s == 0 && e0 != 0)) {
      atomicOr(&ctrl->status, ERR_LP_LIST);
    } else {
      const uint64_t H = off[hp + 1] - off[hp];
      const uint64_t want = H > 0 ? H - 1 : 0;
      if (gap_off[s + 1] < gap_off[s] || gap_off[s + 1] - gap_off[s] != want || (s == 0 && gap_off[0] != 0))
        atomicOr(&ctrl->status, ERR_GAP_OFFSETS);
      atomicOr(&role[hp], ROLE_HP);
      k_here = static_cast<uint32_t>(e1 - e0);
      uint64_t launches = 0;
      for (uint64_t e = e0; e < e1; ++e) {
        const uint32_t lp = lp_task[e], q = lp_prio[e];
        if (lp >= n_tasks) { atomicOr(&ctrl->status, ERR_TASK_INDEX); continue; }
        if (q < 1 || q > 9) atomicOr(&ctrl->status, ERR_LP_LIST);
        launches += off[lp + 1] - off[lp];
        atomicOr(&role[lp], ROLE_LP);
      }
      // (the age of a waiting request is counted in 32 bits: one tick per list entry, then one per kernel issued)
      if (launches + (e1 - e0) >= (1ull << 32)) atomicOr(&ctrl->status, ERR_LP_LIMIT);
    }
  }
  const uint32_t k_wave = wave_max_u32(k_here);
  if (lane_id() == 0 && k_wave) atomicMax(&ctrl->n_class[3], k_wave);
}

constexpr int PW_THREADS = 128;
constexpr uint32_t PW_OPENS = 3, PW_TRIES = 6;   // per period: gaps opened, and decisions per gap opened
static_assert(2 * PW_OPENS + 7 < 16, "the staged results of a period fit the ring");
constexpr uint32_t PW_OUT_CAP = 16;              // staged results: at most 7 left over + 2 per gap opened in a period

template <int W>
struct PrioWalkSmem {   // [entry][column]: a lane's durations in its own column; the idle times and the results of a
                        // scenario in the column of its group
  uint32_t lp[LW_LP_CAP][PW_THREADS];
  uint32_t hp_g[LW_HP_CAP][PW_THREADS / W];
  uint32_t out_c[PW_OUT_CAP][PW_THREADS / W];
  uint32_t out_f[PW_OUT_CAP][PW_THREADS / W];
};

// Largest value among the W adjacent lanes of a group, in all of them.  Inside a row of 16 lanes the
// values move by data-parallel-primitive swaps (pairs, quads) and mirrors (8, 16 lanes: once all lanes of
// each half hold the half's result, mirroring exchanges the halves); every lane has a source lane in
// these patterns.  All 64 lanes must call.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move(uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ uint32_t max_u32(uint32_t a, uint32_t b) { return a > b ? a : b; }
template <int W>
__device__ __forceinline__ uint32_t group_max_u32(uint32_t v) {
  if (W >= 2) v = max_u32(v, dpp_move<0xB1>(v));    // quad_perm [1,0,3,2]
  if (W >= 4) v = max_u32(v, dpp_move<0x4E>(v));    // quad_perm [2,3,0,1]
  if (W >= 8) v = max_u32(v, dpp_move<0x141>(v));   // row_half_mirror
  if (W >= 16) v = max_u32(v, dpp_move<0x140>(v));  // row_mirror
  if (W >= 32) v = max_u32(v, static_cast<uint32_t>(__shfl_xor(v, 16, WAVE)));
  if (W >= 64) v = max_u32(v, static_cast<uint32_t>(__shfl_xor(v, 32, WAVE)));
  return v;
}

// What a lane offers to a decision (the largest offer of the group decides what happens):
enum : uint32_t {
  OFFER_NONE = 0,    // the lane has no request left
  OFFER_NO_FIT = 1,  // its request is longer than what is left of the gap
  // 15 - level (6 .. 14): its request fits
  OFFER_WAIT = 15,   // its request is not known yet (still being read): nothing is decided in this step
};

template <int W>
__device__ __forceinline__ void pw_store_scalar(const PrioWalkSmem<W>& sm, uint32_t col, uint32_t first, uint32_t count,
                                                uint32_t* __restrict__ fill_count, int64_t* __restrict__ filled_ns) {
  for (uint32_t k = 0; k < count; ++k) {
    const uint32_t at = first + k;
    fill_count[at] = sm.out_c[at & (PW_OUT_CAP - 1)][col];
    filled_ns[at] = static_cast<int64_t>(sm.out_f[at & (PW_OUT_CAP - 1)][col]);
  }
}

// W adjacent lanes (a power of two, W <= 64) step through one scenario together.  Every lane owns one
// low-priority task: a ring of its next predicted durations, the position of its waiting request and
// when that request was enqueued.  The first lane of the group also owns the ring of predicted idle
// times of the high-priority trace and writes the per-gap results; what describes the open gap (time
// left, kernels issued, time filled) is kept identically in all lanes of the group.
// One BestPrioFit decision, three reductions over the group: the highest level among the lanes whose
// request fits (and whether any request is still unknown, does not fit, or is left at all); the longest
// duration among those lanes; the longest wait among the lanes that offer it.  That lane's request is
// issued and its next request enqueued.  With W == 1 this is the first-in-first-out walk of one queue.
template <int W>
__global__ void __launch_bounds__(PW_THREADS)
k_pf_walk(const uint64_t* __restrict__ off, const uint32_t* __restrict__ hp_task, const uint64_t* __restrict__ lp_off,
          const uint32_t* __restrict__ lp_task, const uint32_t* __restrict__ lp_prio, uint64_t n_scen,
          const uint64_t* __restrict__ gap_off, const uint32_t* __restrict__ lp_e, const uint2* __restrict__ hp_eg,
          int64_t margin, int64_t min_gap, uint32_t* __restrict__ fill_count, int64_t* __restrict__ filled_ns,
          uint64_t* __restrict__ placed_out, int64_t* __restrict__ placed_ns_out, uint32_t vec_ok, const Ctrl* ctrl) {
  static_assert(W >= 1 && W <= WAVE && (W & (W - 1)) == 0, "group width");
  extern __shared__ __align__(16) unsigned char pw_raw[];
  PrioWalkSmem<W>& sm = *reinterpret_cast<PrioWalkSmem<W>*>(pw_raw);
  if (ctrl->status || ctrl->wide) return;
  const uint32_t tid = threadIdx.x;
  const uint32_t member = tid & (W - 1);
  const uint32_t col = tid / W;                            // column of the group's shared rings
  const uint64_t s = (static_cast<uint64_t>(blockIdx.x) * PW_THREADS + tid) / W;
  const bool valid = s < n_scen;
  const bool lead = valid && member == 0;
  const uint32_t gshift = lane_id() & ~static_cast<uint32_t>(W - 1);
  const uint64_t gmask = W == WAVE ? ~0ull : ((1ull << (W & 63)) - 1ull) << gshift;

  // positions are global element numbers (all below 2^32)
  uint32_t h0 = 0, hp_end = 0, l0 = 0, lp_end = 0, g_first = 0, n_gaps = 0, prio = 0;
  uint64_t entry = 0;
  bool has_entry = false;
  if (valid) {
    const uint32_t hp = hp_task[s];
    h0 = static_cast<uint32_t>(off[hp]); hp_end = static_cast<uint32_t>(off[hp + 1]);
    g_first = static_cast<uint32_t>(gap_off[s]);
    n_gaps = hp_end > h0 ? hp_end - h0 - 1 : 0;
    const uint64_t e0 = lp_off[s], K = lp_off[s + 1] - e0;
    if (member < K) {
      entry = e0 + member;
      const uint32_t lp = lp_task[entry];
      l0 = static_cast<uint32_t>(off[lp]); lp_end = static_cast<uint32_t>(off[lp + 1]);
      prio = lp_prio[entry];
      has_entry = true;
    }
  }
  uint32_t hp_pos = h0, lp_pos = l0;
  uint32_t hp_landed = h0 & ~(LW_HP_CHUNK - 1), lp_landed = l0 & ~(LW_LP_CHUNK - 1);   // rings hold entries below these
  uint32_t hp_req = 0, lp_req = 0;
  bool hp_fly = false, lp_fly = false;
  uint4 hr[4], lr[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) hr[k] = lr[k] = make_uint4(0, 0, 0, 0);

  uint32_t g = g_first;              // global number of the next gap to report
  uint32_t flushed = g_first;        // results below this are in memory
  const uint32_t g_end = g_first + n_gaps;
  uint32_t c = 0, f = 0, rem = 0;
  const uint32_t offer_fit = 15u - prio;
  uint32_t clock = W;                // enqueue stamps handed out so far (only their order matters: the initial
  uint32_t stamp = member;           // requests are enqueued in list order, before everything else)
  uint64_t placed_ns = 0;
  const int64_t floor64 = min_gap > margin ? min_gap : margin;
  const uint32_t gap_floor = floor64 >= static_cast<int64_t>(WIDE32) ? WIDE32 : static_cast<uint32_t>(floor64);
  const uint32_t margin32 = margin >= static_cast<int64_t>(WIDE32) ? WIDE32 : static_cast<uint32_t>(margin);
  bool in_gap = false;
  bool pending = false;               // a gap has closed and its result (c, f) is not staged yet
  // nothing to step through: no scenario, or no low-priority kernel at all (every gap then gets zeros)
  const bool no_kernels = (ballot(lp_end == l0) & gmask) == gmask;
  bool finished = !valid || no_kernels;

  for (;;) {
    // ---- once per period: park what was read, read on, write complete groups of results ----
    if (hp_fly) {
      if (lead) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const uint32_t at = (hp_req + 2 * k) & (LW_HP_CAP - 1);
          sm.hp_g[at][col] = hr[k].y;
          sm.hp_g[at + 1][col] = hr[k].w;
        }
      }
      hp_landed = hp_req + LW_HP_CHUNK;
      hp_fly = false;
    }
    if (lp_fly) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t at = (lp_req + 4 * k) & (LW_LP_CAP - 1);
        sm.lp[at][tid] = lr[k].x; sm.lp[at + 1][tid] = lr[k].y; sm.lp[at + 2][tid] = lr[k].z; sm.lp[at + 3][tid] = lr[k].w;
      }
      lp_landed = lp_req + LW_LP_CHUNK;
      lp_fly = false;
    }
    if (!finished && hp_landed < hp_end && static_cast<int32_t>(hp_landed - hp_pos) <= static_cast<int32_t>(LW_HP_CAP - LW_HP_CHUNK)) {
      if (lead) {
        const uint4* src = reinterpret_cast<const uint4*>(hp_eg + hp_landed);
#pragma unroll
        for (int k = 0; k < 4; ++k) hr[k] = src[k];
      }
      hp_req = hp_landed;
      hp_fly = true;
    }
    if (!finished && lp_landed < lp_end && static_cast<int32_t>(lp_landed - lp_pos) <= static_cast<int32_t>(LW_LP_CAP - LW_LP_CHUNK)) {
      const uint4* src = reinterpret_cast<const uint4*>(lp_e + lp_landed);
#pragma unroll
      for (int k = 0; k < 4; ++k) lr[k] = src[k];
      lp_req = lp_landed;
      lp_fly = true;
    }
    if (flushed < g && (flushed & (LW_OUT_CHUNK - 1))) {   // (first results of a scenario, up to a multiple of 8)
      const uint32_t to8 = LW_OUT_CHUNK - (flushed & (LW_OUT_CHUNK - 1));
      const uint32_t cnt = g - flushed < to8 ? g - flushed : to8;
      if (lead) pw_store_scalar<W>(sm, col, flushed, cnt, fill_count, filled_ns);
      flushed += cnt;
    }
    while (flushed + LW_OUT_CHUNK <= g) {
      if (lead) {
        if (vec_ok) {
          const uint32_t at = flushed & (PW_OUT_CAP - 1);
          uint32_t cc[LW_OUT_CHUNK], ff[LW_OUT_CHUNK];
#pragma unroll
          for (uint32_t k = 0; k < LW_OUT_CHUNK; ++k) { cc[k] = sm.out_c[at + k][col]; ff[k] = sm.out_f[at + k][col]; }
          uint4* oc = reinterpret_cast<uint4*>(fill_count + flushed);
          oc[0] = make_uint4(cc[0], cc[1], cc[2], cc[3]);
          oc[1] = make_uint4(cc[4], cc[5], cc[6], cc[7]);
          uint4* of = reinterpret_cast<uint4*>(filled_ns + flushed);
#pragma unroll
          for (uint32_t k = 0; k < 4; ++k) of[k] = make_uint4(ff[2 * k], 0u, ff[2 * k + 1], 0u);
        } else {
          pw_store_scalar<W>(sm, col, flushed, LW_OUT_CHUNK, fill_count, filled_ns);
        }
      }
      flushed += LW_OUT_CHUNK;
    }
    if (__all(finished)) break;

    // ---- one period, without branches: PW_OPENS times { stage the result of the gap that closed, take
    // the next high-priority launch and open its gap; PW_TRIES decisions }.  A group whose rings lack an
    // entry it needs idles in that sub-step. ----
#pragma unroll
    for (uint32_t o = 0; o < PW_OPENS; ++o) {
      {
        // (a staging slot that is written early is simply written again; all lanes of a group write the same)
        sm.out_c[g & (PW_OUT_CAP - 1)][col] = c;
        sm.out_f[g & (PW_OUT_CAP - 1)][col] = f;
        g += pending ? 1u : 0u;
        pending = false;
        const uint32_t G = sm.hp_g[hp_pos & (LW_HP_CAP - 1)][col];
        // between gaps: the next high-priority launch runs, then its gap opens (the last launch has none)
        const bool idle = !finished && !in_gap;
        const bool at_end = idle && hp_pos == hp_end;
        const bool take = idle && !at_end && hp_pos < hp_landed;
        hp_pos += take ? 1u : 0u;
        const bool last = take && hp_pos == hp_end;
        const bool gap = take && !last;
        const bool usable = gap && G >= gap_floor;
        const bool skip = gap && !usable;
        // a skipped gap reports zeros
        sm.out_c[g & (PW_OUT_CAP - 1)][col] = 0u;
        sm.out_f[g & (PW_OUT_CAP - 1)][col] = 0u;
        g += skip ? 1u : 0u;
        in_gap = in_gap || usable;
        rem = usable ? G - margin32 : rem;
        c = usable ? 0u : c;
        f = usable ? 0u : f;
        finished = finished || at_end || last;
      }
#pragma unroll
      for (uint32_t k = 0; k < PW_TRIES; ++k) {
        const uint32_t d = sm.lp[lp_pos & (LW_LP_CAP - 1)][tid];
        const uint32_t offer = lp_pos == lp_end ? OFFER_NONE                    // (also: a lane without a task)
                               : lp_pos >= lp_landed ? OFFER_WAIT
                               : d <= rem ? offer_fit : OFFER_NO_FIT;
        const uint32_t top = group_max_u32<W>(offer);                           // (all lanes take part)
        const uint32_t best = in_gap ? top : OFFER_WAIT;
        const bool any = best - 6u <= 8u;                                       // some request fits: best = 15 - its level
        const bool at_level = any && offer == best;
        const uint32_t longest = group_max_u32<W>(at_level ? d + 1u : 0u);      // (durations are below 2^32 - 1)
        const bool tie = at_level && d + 1u == longest;
        const uint32_t age = tie ? clock - stamp : 0u;                          // >= 1 for a waiting request
        const uint32_t oldest = group_max_u32<W>(age);
        const bool win = tie && age == oldest;
        const uint32_t dd = any ? longest - 1u : 0u;
        rem -= dd; f += dd;
        c += any ? 1u : 0u;
        lp_pos += win ? 1u : 0u;
        placed_ns += win ? dd : 0u;
        stamp = win ? clock : stamp;                             // the task's following kernel is enqueued now
        clock += any ? 1u : 0u;
        // nothing fits: the gap is done; no request left anywhere (seen one decision after the last issue):
        // so is the scenario
        const bool close = best <= OFFER_NO_FIT;
        pending = pending || close;
        finished = finished || best == OFFER_NONE;
        in_gap = in_gap && !close;
      }
    }
  }

  if (!valid) return;
  if (pending) {
    sm.out_c[g & (PW_OUT_CAP - 1)][col] = c;
    sm.out_f[g & (PW_OUT_CAP - 1)][col] = f;
    ++g;
  }
  if (has_entry) {
    placed_out[entry] = lp_pos - l0;
    placed_ns_out[entry] = static_cast<int64_t>(placed_ns);
  }
  if (!lead) return;
  // what is still staged, then zeros for the gaps after the queues ran empty
  pw_store_scalar<W>(sm, col, flushed, g - flushed, fill_count, filled_ns);
  uint32_t z = g;
  while (z < g_end && (z & (LW_OUT_CHUNK - 1))) { fill_count[z] = 0; filled_ns[z] = 0; ++z; }
  if (vec_ok) {
    for (; z + LW_OUT_CHUNK <= g_end; z += LW_OUT_CHUNK) {
      uint4* oc = reinterpret_cast<uint4*>(fill_count + z);
      oc[0] = oc[1] = make_uint4(0, 0, 0, 0);
      uint4* of = reinterpret_cast<uint4*>(filled_ns + z);
      of[0] = of[1] = of[2] = of[3] = make_uint4(0, 0, 0, 0);
    }
  }
  for (; z < g_end; ++z) { fill_count[z] = 0; filled_ns[z] = 0; }
}

// Algorithm 1 with the whole of Algorithm 2 for the scenarios the group kernels do not take: predictions that do not
// fit 32 bits (Ctrl::wide), or more low-priority tasks in a scenario than a wave has lanes.  One lane per scenario
// steps through the gaps literally on the 64-bit arrays of k_gf_predict; every decision looks at all the scenario's
// waiting requests.  The state of a list entry lives in its own output word while the walk runs: the low half of
// lp_placed counts its kernels issued so far (= the position of its waiting request), the high half is the stamp of
// that request; the high half is cleared at the end.  Rare and slow on purpose.
__global__ void __launch_bounds__(64)
k_pf_walk_wide(const uint64_t* __restrict__ off, const uint32_t* __restrict__ hp_task, const uint64_t* __restrict__ lp_off,
               const uint32_t* __restrict__ lp_task, const uint32_t* __restrict__ lp_prio, uint64_t n_scen,
               const uint64_t* __restrict__ gap_off, const int64_t* __restrict__ pe, const int64_t* __restrict__ pg,
               int64_t margin, int64_t min_gap, uint32_t* __restrict__ fill_count, int64_t* __restrict__ filled_ns,
               uint64_t* __restrict__ placed, int64_t* __restrict__ placed_ns, uint32_t only_if_wide, const Ctrl* ctrl) {
  if (ctrl->status) return;
  if (only_if_wide && !ctrl->wide) return;
  const uint64_t s = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (s >= n_scen) return;
  const uint32_t hp = hp_task[s];
  const uint64_t h0 = off[hp], H = off[hp + 1] - h0;
  const uint64_t e0 = lp_off[s], K = lp_off[s + 1] - e0;
  const uint64_t g0 = gap_off[s];
  for (uint64_t k = 0; k < K; ++k) { placed[e0 + k] = k << 32; placed_ns[e0 + k] = 0; }   // initial requests: enqueued in list order
  uint64_t clock = K;
  // predicted duration of the waiting request of entry k (whose state word is st), or -1 if the task has none left
  auto waiting = [&](uint64_t k, uint64_t st) -> int64_t {
    const uint32_t lp = lp_task[e0 + k];
    const uint64_t l0 = off[lp], L = off[lp + 1] - l0, nxt = st & 0xffffffffull;
    if (nxt >= L) return -1;
    return pe[l0 + nxt] - (nxt ? pe[l0 + nxt - 1] : 0);
  };
  for (uint64_t i = 0; i + 1 < H; ++i) {
    const int64_t G = pg[h0 + i];
    uint32_t c = 0;
    int64_t f = 0;
    if (G >= min_gap && G >= margin) {
      int64_t rem = G - margin;
      for (;;) {
        // BestPrioFit: the highest level with a request that fits; there the longest; among equally long ones the oldest
        bool found = false;
        uint64_t best = 0, best_stamp = 0;
        uint32_t best_level = 0;
        int64_t best_d = 0;
        for (uint64_t k = 0; k < K; ++k) {
          const uint64_t st = placed[e0 + k];
          const int64_t d = waiting(k, st);
          if (d < 0 || d > rem) continue;
          const uint32_t level = lp_prio[e0 + k];
          const uint64_t stamp = st >> 32;
          if (!found || level < best_level || (level == best_level && (d > best_d || (d == best_d && stamp < best_stamp)))) {
            found = true; best = k; best_level = level; best_d = d; best_stamp = stamp;
          }
        }
        if (!found) break;
        rem -= best_d; f += best_d; ++c;
        const uint64_t st = placed[e0 + best];
        placed[e0 + best] = (clock << 32) | ((st & 0xffffffffull) + 1);   // the task's following kernel is enqueued now
        ++clock;
        placed_ns[e0 + best] += best_d;
      }
    }
    fill_count[g0 + i] = c;
    filled_ns[g0 + i] = f;
  }
  for (uint64_t k = 0; k < K; ++k) placed[e0 + k] &= 0xffffffffull;
}

}  // namespace fikit
