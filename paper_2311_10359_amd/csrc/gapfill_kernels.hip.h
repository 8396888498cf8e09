// Gap filling (Algorithm 1, FIKIT procedure; Algorithm 2, BestPrioFit, with a single waiting
// request): per scenario, walk the high-priority trace and issue the low-priority task's next
// kernels into each predicted idle gap for as long as they fit.
//
// Because predicted durations are >= 0, "keep issuing the head of the queue while it fits into
// what is left" is the same as "advance the queue pointer to the last position whose prefix sum
// of durations does not exceed (consumed so far) + (gap - margin)".  The kernels therefore work
// on per-task prefix sums and search them with ballots.
#pragma once

#include "common.hip.h"

namespace fikit {

constexpr uint32_t ROLE_HP = 1u, ROLE_LP = 2u;

// Checks scenario arguments and records in role[t] how each task is used.
__global__ void k_gf_scenarios(const uint64_t* __restrict__ off, uint32_t n_tasks, const uint32_t* __restrict__ hp_task,
                               const uint32_t* __restrict__ lp_task, uint64_t n_scen,
                               const uint64_t* __restrict__ gap_off, uint32_t* __restrict__ role, Ctrl* ctrl) {
  if (ctrl->status & ERR_OFFSETS) return;
  const uint64_t s = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (s >= n_scen) return;
  const uint32_t hp = hp_task[s], lp = lp_task[s];
  if (hp >= n_tasks || lp >= n_tasks) { atomicOr(&ctrl->status, ERR_TASK_INDEX); return; }
  const uint64_t H = off[hp + 1] - off[hp];
  const uint64_t want = H > 0 ? H - 1 : 0;
  if (gap_off[s + 1] < gap_off[s] || gap_off[s + 1] - gap_off[s] != want || (s == 0 && gap_off[0] != 0))
    atomicOr(&ctrl->status, ERR_GAP_OFFSETS);
  atomicOr(&role[hp], ROLE_HP);
  atomicOr(&role[lp], ROLE_LP);
}

// Predicted values of one launch, looked up by Kernel ID in the task's rows (sorted by ID).
struct Pred { int64_t e, g; bool found; };

constexpr int PRED_THREADS = 256;
constexpr int PRED_TABLE = 2048;  // rows of a task kept in LDS for the lookup

// One workgroup per task that takes part in a scenario.  For every launch i of the task:
//   as low-priority queue:   pe[i]   = sum of predicted execution times of launches 0..i
//   as high-priority trace:  pg[i]   = predicted idle time after launch i
//                            open[i] = predicted time at which launch i ends (its gap opens):
//                                      sum_{k<=i} E_k + sum_{k<i} G_k
__global__ void __launch_bounds__(PRED_THREADS)
k_gf_predict(const uint64_t* __restrict__ ids, const uint64_t* __restrict__ off, uint32_t n_tasks,
             const fikit_row* __restrict__ rows, const uint64_t* __restrict__ row_off, const uint32_t* __restrict__ role,
             int64_t* __restrict__ pe, int64_t* __restrict__ pg, int64_t* __restrict__ open, Ctrl* ctrl) {
  __shared__ uint64_t t_key[PRED_TABLE];
  __shared__ int64_t t_e[PRED_TABLE];
  __shared__ int64_t t_g[PRED_TABLE];
  __shared__ uint64_t wsum[2][4];
  // only bits that earlier kernels set: the decision must be the same for the whole workgroup
  if (ctrl->status & (ERR_OFFSETS | ERR_TASK_INDEX | ERR_GAP_OFFSETS)) return;
  const uint32_t t = blockIdx.x;
  const uint32_t rl = role[t];
  if (rl == 0) return;
  const uint64_t base = off[t], len = off[t + 1] - base;
  const uint64_t r0 = row_off[t], nr = row_off[t + 1] - r0;
  const uint32_t tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const bool in_lds = nr <= PRED_TABLE;
  if (in_lds) {
    for (uint32_t r = tid; r < nr; r += PRED_THREADS) {
      const fikit_row* row = rows + r0 + r;
      t_key[r] = row->kernel_id;
      t_e[r] = row->exec.p50;
      t_g[r] = row->gap.p50;
    }
  }
  __syncthreads();
  uint64_t carry_e = 0, carry_o = 0;  // sums over all earlier launches: E, and E + G
  for (uint64_t c0 = 0; c0 < len; c0 += PRED_THREADS) {
    const uint64_t i = c0 + tid;
    int64_t e = 0, g = 0;
    if (i < len) {
      const uint64_t id = ids[base + i];
      // lower bound in the task's sorted IDs
      uint64_t lo = 0, hi = nr;
      if (in_lds) {
        while (lo < hi) { const uint64_t mid = (lo + hi) >> 1; if (t_key[mid] < id) lo = mid + 1; else hi = mid; }
        if (lo < nr && t_key[lo] == id) { e = t_e[lo]; g = t_g[lo]; } else atomicOr(&ctrl->status, ERR_UNKNOWN_ID);
      } else {
        while (lo < hi) { const uint64_t mid = (lo + hi) >> 1; if (rows[r0 + mid].kernel_id < id) lo = mid + 1; else hi = mid; }
        if (lo < nr && rows[r0 + lo].kernel_id == id) { e = rows[r0 + lo].exec.p50; g = rows[r0 + lo].gap.p50; }
        else atomicOr(&ctrl->status, ERR_UNKNOWN_ID);
      }
    }
    const uint64_t ue = static_cast<uint64_t>(e), uo = static_cast<uint64_t>(e) + static_cast<uint64_t>(g);
    const uint64_t ie = wave_incl_scan_u64(ue), io = wave_incl_scan_u64(uo);
    __syncthreads();
    if (lane == 63) { wsum[0][w] = ie; wsum[1][w] = io; }
    __syncthreads();
    uint64_t be = carry_e, bo = carry_o;
    for (uint32_t k = 0; k < w; ++k) { be += wsum[0][k]; bo += wsum[1][k]; }
    if (i < len) {
      if (rl & ROLE_LP) pe[base + i] = static_cast<int64_t>(be + ie);
      if (rl & ROLE_HP) {
        pg[base + i] = g;
        open[base + i] = static_cast<int64_t>(bo + io - static_cast<uint64_t>(g));
      }
    }
    carry_e += wsum[0][0] + wsum[0][1] + wsum[0][2] + wsum[0][3];
    carry_o += wsum[1][0] + wsum[1][1] + wsum[1][2] + wsum[1][3];
  }
}

// The walk.  GW lanes cooperate on one scenario (GW divides 64): they read GW predicted gaps
// at a time, and search the low-priority prefix sums GW candidates at a time with a ballot.
template <int GW>
__global__ void __launch_bounds__(256)
k_gf_walk(const uint64_t* __restrict__ off, const uint32_t* __restrict__ hp_task, const uint32_t* __restrict__ lp_task,
          uint64_t n_scen, const uint64_t* __restrict__ gap_off, const int64_t* __restrict__ pe,
          const int64_t* __restrict__ pg, const int64_t* __restrict__ open, int64_t margin, int64_t min_gap,
          uint32_t* __restrict__ fill_count, int64_t* __restrict__ filled_ns, int64_t* __restrict__ completion_out,
          uint64_t* __restrict__ placed_out, const Ctrl* ctrl) {
  if (ctrl->status) return;
  constexpr int GROUPS_PER_BLOCK = 256 / GW;
  const uint64_t s = static_cast<uint64_t>(blockIdx.x) * GROUPS_PER_BLOCK + threadIdx.x / GW;
  if (s >= n_scen) return;  // whole groups leave together
  const uint32_t lane = lane_id();
  const uint32_t gl = lane % GW;           // lane within the group
  const uint32_t gbase = lane - gl;        // first lane of the group
  const uint64_t gmask = (GW == 64) ? ~0ull : ((1ull << GW) - 1ull);

  const uint32_t hp = hp_task[s], lp = lp_task[s];
  const uint64_t h0 = off[hp], H = off[hp + 1] - h0;
  const uint64_t l0 = off[lp], L = off[lp + 1] - l0;
  const uint64_t g0 = gap_off[s];
  const uint64_t n_gaps = H > 0 ? H - 1 : 0;

  uint64_t p = 0;         // low-priority kernels issued so far
  int64_t consumed = 0;   // their total predicted duration = pe[l0 + p - 1]
  bool done = (L == 0);
  int64_t completion = 0;

  for (uint64_t i0 = 0; i0 < n_gaps; i0 += GW) {
    const uint64_t mine = i0 + gl;
    const int64_t my_g = mine < n_gaps ? pg[h0 + mine] : 0;
    uint32_t my_c = 0;
    int64_t my_f = 0;
    const uint32_t steps = static_cast<uint32_t>(n_gaps - i0 < GW ? n_gaps - i0 : GW);
    for (uint32_t k = 0; k < steps; ++k) {
      const int64_t G = static_cast<int64_t>(shfl_u64(static_cast<uint64_t>(my_g), gbase + k));
      uint32_t c = 0;
      int64_t f = 0;
      if (G >= min_gap && G >= margin && p < L) {
        const int64_t limit = consumed + (G - margin);
        int64_t last_fit = consumed;
        for (;;) {
          const uint64_t j = p + c + gl;
          const int64_t val = j < L ? pe[l0 + j] : INT64_MAX;
          const bool fits = (j < L) && (val <= limit);
          const uint64_t b = (ballot(fits) >> gbase) & gmask;
          const uint32_t cnt = (b == gmask) ? GW : static_cast<uint32_t>(__builtin_ctzll(~b));
          if (cnt > 0) last_fit = static_cast<int64_t>(shfl_u64(static_cast<uint64_t>(val), gbase + cnt - 1));
          c += cnt;
          if (cnt < GW) break;
        }
        f = last_fit - consumed;
        consumed = last_fit;
        p += c;
        if (p == L && c > 0 && !done) {
          completion = open[h0 + i0 + k] + f;
          done = true;
        }
      }
      if (gl == k) { my_c = c; my_f = f; }
    }
    if (mine < n_gaps) {
      fill_count[g0 + mine] = my_c;
      filled_ns[g0 + mine] = my_f;
    }
  }
  if (!done) {
    const int64_t t_end = H > 0 ? open[h0 + H - 1] : 0;
    const int64_t rest = L > 0 ? pe[l0 + L - 1] - consumed : 0;
    completion = t_end + rest;
  }
  if (gl == 0) {
    completion_out[s] = completion;
    placed_out[s] = p;
  }
}

}  // namespace fikit
