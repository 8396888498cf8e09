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

// Checks scenario arguments (n_gaps: the number of per-gap output slots the host sized its buffers for) and
// records in role[t] how each task is used.
__global__ void k_gf_scenarios(const uint64_t* __restrict__ off, uint32_t n_tasks, const uint32_t* __restrict__ hp_task,
                               const uint32_t* __restrict__ lp_task, uint64_t n_scen,
                               const uint64_t* __restrict__ gap_off, uint64_t n_gaps, uint32_t* __restrict__ role, Ctrl* ctrl) {
  if (ctrl->status & ERR_OFFSETS) return;
  const uint64_t s = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (s >= n_scen) return;
  if (s + 1 == n_scen && gap_off[n_scen] != n_gaps) atomicOr(&ctrl->status, ERR_GAP_OFFSETS);
  const uint32_t hp = hp_task[s], lp = lp_task[s];
  if (hp >= n_tasks || lp >= n_tasks) { atomicOr(&ctrl->status, ERR_TASK_INDEX); return; }
  const uint64_t H = off[hp + 1] - off[hp];
  const uint64_t want = H > 0 ? H - 1 : 0;
  if (gap_off[s + 1] < gap_off[s] || gap_off[s + 1] - gap_off[s] != want || (s == 0 && gap_off[0] != 0))
    atomicOr(&ctrl->status, ERR_GAP_OFFSETS);
  atomicOr(&role[hp], ROLE_HP);
  atomicOr(&role[lp], ROLE_LP);
}

// Work list of the predict kernel: tasks that play a role, short traces first, long ones after, so
// that workgroups started next to each other have work of similar size.
__global__ void k_gf_lists(const uint64_t* __restrict__ off, uint32_t n_tasks, const uint32_t* __restrict__ role,
                           uint32_t split_len, uint32_t* __restrict__ lists, Ctrl* ctrl) {
  if (ctrl->status & (ERR_OFFSETS | ERR_TASK_INDEX | ERR_GAP_OFFSETS)) return;
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  uint32_t c = 2;
  if (t < n_tasks && role[t]) c = (off[t + 1] - off[t]) <= split_len ? 0u : 1u;
  for (uint32_t k = 0; k < 2; ++k) {
    const uint32_t pos = wave_append(&ctrl->n_class[k], c == k);
    if (c == k) lists[static_cast<uint64_t>(k) * n_tasks + pos] = static_cast<uint32_t>(t);
  }
}

constexpr int PRED_THREADS = 256;
constexpr int PRED_KPT = 8;                       // consecutive launches per thread and chunk
constexpr int PRED_CHUNK = PRED_THREADS * PRED_KPT;
constexpr int PRED_ROWS = 512;                    // rows of a task kept in an LDS hash table for the lookup
constexpr int PRED_HT = 2 * PRED_ROWS;

// The prediction read from a row's statistics: median, or mean = sum / count (Section 3.2: SK_j, SG_j).
__device__ __forceinline__ int64_t predicted_of(const fikit_stats& st, uint32_t predictor) {
  if (predictor == FIKIT_PREDICT_P50) return st.p50;
  return st.count ? static_cast<int64_t>(st.sum / st.count) : 0;
}

// Predicted execution time and idle time of a launch: taken from its ID's row.  Rows of a
// task with few IDs sit in an LDS hash table keyed by the ID; otherwise the task's sorted rows
// are searched in memory.
struct PredTable {
  uint64_t key[PRED_HT];
  int64_t e[PRED_HT];
  int64_t g[PRED_HT];
};

__device__ __forceinline__ bool predict_one(uint64_t id, bool in_lds, const PredTable& tb, const fikit_row* __restrict__ rows,
                                            uint64_t r0, uint64_t nr, uint32_t predictor, int64_t& e, int64_t& g) {
  if (in_lds) {
    uint32_t h = (static_cast<uint32_t>(id >> 32) ^ static_cast<uint32_t>(id)) & (PRED_HT - 1);
    for (int probe = 0; probe < PRED_HT; ++probe) {
      const uint64_t k = tb.key[h];
      if (k == id) { e = tb.e[h]; g = tb.g[h]; return true; }
      if (k == ~0ull) return false;
      h = (h + 1) & (PRED_HT - 1);
    }
    return false;
  }
  uint64_t lo = 0, hi = nr;
  while (lo < hi) { const uint64_t mid = (lo + hi) >> 1; if (rows[r0 + mid].kernel_id < id) lo = mid + 1; else hi = mid; }
  if (lo < nr && rows[r0 + lo].kernel_id == id) {
    e = predicted_of(rows[r0 + lo].exec, predictor);
    g = predicted_of(rows[r0 + lo].gap, predictor);
    return true;
  }
  return false;
}

// One workgroup per task that takes part in a scenario.  For every launch i of the task:
//   as low-priority queue:   pe[i]   = sum of predicted execution times of launches 0..i
//   as high-priority trace:  pg[i]   = predicted idle time after launch i
//                            open[i] = predicted time at which launch i ends (its gap opens):
//                                      sum_{k<=i} E_k + sum_{k<i} G_k   (not written if open is null)
// Prefix sums run thread -> wave -> workgroup, with a running carry from chunk to chunk.
__global__ void __launch_bounds__(PRED_THREADS) __attribute__((amdgpu_waves_per_eu(5, 8)))
k_gf_predict(const uint64_t* __restrict__ ids, const uint64_t* __restrict__ off, uint32_t n_tasks,
             const fikit_row* __restrict__ rows, const uint64_t* __restrict__ row_off, const uint32_t* __restrict__ role,
             const uint32_t* __restrict__ lists, int64_t* __restrict__ pe, int64_t* __restrict__ pg,
             int64_t* __restrict__ open, uint32_t only_if_wide, uint32_t predictor, Ctrl* ctrl) {
  __shared__ PredTable tb;
  // only bits that earlier kernels set: the decision must be the same for the whole workgroup
  if (ctrl->status & (ERR_OFFSETS | ERR_TASK_INDEX | ERR_GAP_OFFSETS)) return;
  if (only_if_wide && !ctrl->wide) return;
  const uint32_t n_short = ctrl->n_class[0], n_longer = ctrl->n_class[1];   // final: set by an earlier kernel
  if (blockIdx.x >= n_short + n_longer) return;
  const uint32_t t = blockIdx.x < n_short ? lists[blockIdx.x] : lists[static_cast<uint64_t>(n_tasks) + (blockIdx.x - n_short)];
  const uint32_t rl = role[t];
  if (rl == 0) return;
  const uint64_t base = off[t], len = off[t + 1] - base;
  const uint64_t r0 = row_off[t], nr = row_off[t + 1] - r0;
  const uint32_t tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  // (an ID equal to the table's "empty" mark can only be the largest one)
  const bool in_lds = nr <= PRED_ROWS && (nr == 0 || rows[r0 + nr - 1].kernel_id != ~0ull);
  if (in_lds) {
    for (uint32_t h = tid; h < PRED_HT; h += PRED_THREADS) tb.key[h] = ~0ull;
    __syncthreads();
    for (uint32_t r = tid; r < nr; r += PRED_THREADS) {
      const fikit_row* row = rows + r0 + r;
      const uint64_t id = row->kernel_id;
      uint32_t h = (static_cast<uint32_t>(id >> 32) ^ static_cast<uint32_t>(id)) & (PRED_HT - 1);
      for (;;) {   // IDs of a task are distinct and fill at most half the table: a free slot exists
        const uint64_t old = atomicCAS(reinterpret_cast<unsigned long long*>(&tb.key[h]), ~0ull, id);
        if (old == ~0ull) break;
        h = (h + 1) & (PRED_HT - 1);
      }
      tb.e[h] = predicted_of(row->exec, predictor);
      tb.g[h] = predicted_of(row->gap, predictor);
    }
  }
  __syncthreads();
  uint64_t carry_e = 0, carry_o = 0;  // sums over all earlier launches: E, and E + G
  bool unknown = false;
  // A chunk is PRED_SUB sub-chunks of 2 * PRED_THREADS launches; in a sub-chunk every thread owns
  // two neighbouring launches, so that a wave reads and writes 1 KiB of consecutive memory per access.
  constexpr int PRED_SUB = PRED_KPT / 2;
  __shared__ uint64_t sub_sum[2][PRED_SUB * 4];
  const bool even = ((base & 1) == 0);   // 16-byte accesses to the workspace arrays need an even first index
  const bool ids_vec = (reinterpret_cast<uintptr_t>(ids + base) & 15) == 0;   // and those to the caller's IDs an aligned address
  for (uint64_t c0 = 0; c0 < len; c0 += PRED_CHUNK) {
    int64_t e[PRED_KPT], g[PRED_KPT];
    uint64_t ie[PRED_SUB], io[PRED_SUB];
#pragma unroll
    for (int k = 0; k < PRED_SUB; ++k) {
      const uint64_t i0 = c0 + static_cast<uint64_t>(k) * (2 * PRED_THREADS) + 2 * tid;
      uint64_t id0 = 0, id1 = 0;
      if (ids_vec && i0 + 1 < len) {
        const ulonglong2 v = *reinterpret_cast<const ulonglong2*>(ids + base + i0);
        id0 = v.x; id1 = v.y;
      } else {
        if (i0 < len) id0 = ids[base + i0];
        if (i0 + 1 < len) id1 = ids[base + i0 + 1];
      }
      e[2 * k] = e[2 * k + 1] = g[2 * k] = g[2 * k + 1] = 0;
      if (i0 < len) unknown |= !predict_one(id0, in_lds, tb, rows, r0, nr, predictor, e[2 * k], g[2 * k]);
      if (i0 + 1 < len) unknown |= !predict_one(id1, in_lds, tb, rows, r0, nr, predictor, e[2 * k + 1], g[2 * k + 1]);
      const uint64_t se = static_cast<uint64_t>(e[2 * k]) + static_cast<uint64_t>(e[2 * k + 1]);
      const uint64_t so = se + static_cast<uint64_t>(g[2 * k]) + static_cast<uint64_t>(g[2 * k + 1]);
      // a task needs the sums of the role it plays only (the branch is the same for the whole workgroup)
      ie[k] = io[k] = 0;
      if (rl & ROLE_LP) { ie[k] = wave_incl_scan_u64(se); if (lane == 63) sub_sum[0][k * 4 + w] = ie[k]; ie[k] -= se; }
      if (rl & ROLE_HP) { io[k] = wave_incl_scan_u64(so); if (lane == 63) sub_sum[1][k * 4 + w] = io[k]; io[k] -= so; }
    }
    __syncthreads();
    uint64_t run_e = carry_e, run_o = carry_o;
#pragma unroll
    for (int k = 0; k < PRED_SUB; ++k) {
      uint64_t be = run_e, bo = run_o;
#pragma unroll
      for (int ww = 0; ww < 4; ++ww) {
        const uint64_t te = (rl & ROLE_LP) ? sub_sum[0][k * 4 + ww] : 0, to = (rl & ROLE_HP) ? sub_sum[1][k * 4 + ww] : 0;
        if (static_cast<uint32_t>(ww) < w) { be += te; bo += to; }
        run_e += te; run_o += to;
      }
      be += ie[k]; bo += io[k];
      const uint64_t i0 = c0 + static_cast<uint64_t>(k) * (2 * PRED_THREADS) + 2 * tid;
      const uint64_t pe0 = be + static_cast<uint64_t>(e[2 * k]), pe1 = pe0 + static_cast<uint64_t>(e[2 * k + 1]);
      const uint64_t op0 = bo + static_cast<uint64_t>(e[2 * k]);   // E and G of earlier launches + own E
      const uint64_t op1 = op0 + static_cast<uint64_t>(g[2 * k]) + static_cast<uint64_t>(e[2 * k + 1]);
      if (even && i0 + 1 < len) {
        if (rl & ROLE_LP) *reinterpret_cast<ulonglong2*>(pe + base + i0) = make_ulonglong2(pe0, pe1);
        if (rl & ROLE_HP) {
          *reinterpret_cast<ulonglong2*>(pg + base + i0) = make_ulonglong2(static_cast<uint64_t>(g[2 * k]), static_cast<uint64_t>(g[2 * k + 1]));
          if (open) *reinterpret_cast<ulonglong2*>(open + base + i0) = make_ulonglong2(op0, op1);
        }
      } else {
        if (i0 < len) {
          if (rl & ROLE_LP) pe[base + i0] = static_cast<int64_t>(pe0);
          if (rl & ROLE_HP) { pg[base + i0] = g[2 * k]; if (open) open[base + i0] = static_cast<int64_t>(op0); }
        }
        if (i0 + 1 < len) {
          if (rl & ROLE_LP) pe[base + i0 + 1] = static_cast<int64_t>(pe1);
          if (rl & ROLE_HP) { pg[base + i0 + 1] = g[2 * k + 1]; if (open) open[base + i0 + 1] = static_cast<int64_t>(op1); }
        }
      }
    }
    carry_e = run_e;
    carry_o = run_o;
    __syncthreads();   // sub_sum is rewritten by the next chunk
  }
  if (unknown) atomicOr(&ctrl->status, ERR_UNKNOWN_ID);
}

// The walk.  GW lanes cooperate on one scenario (GW divides 64): they read GW predicted gaps
// at a time, and search the low-priority prefix sums GW candidates at a time with a ballot.
// A value of the group's lane `idx`, where idx is the same in all lanes of the group (a whole wave: scalar lane select).
template <int GW>
__device__ __forceinline__ int64_t group_value(int64_t v, uint32_t gbase, uint32_t idx) {
  if constexpr (GW == WAVE) return static_cast<int64_t>(read_lane_u64(static_cast<uint64_t>(v), idx));
  else return static_cast<int64_t>(shfl_u64(static_cast<uint64_t>(v), gbase + idx));
}

template <int GW, bool WINDOW>
__global__ void __launch_bounds__(256)
k_gf_walk(const uint64_t* __restrict__ off, const uint32_t* __restrict__ hp_task, const uint32_t* __restrict__ lp_task,
          uint64_t n_scen, const uint64_t* __restrict__ gap_off, const int64_t* __restrict__ pe,
          const int64_t* __restrict__ pg, const int64_t* __restrict__ open, int64_t margin, int64_t min_gap,
          uint32_t* __restrict__ fill_count, int64_t* __restrict__ filled_ns, int64_t* __restrict__ completion_out,
          uint64_t* __restrict__ placed_out, uint32_t only_if_wide, const Ctrl* ctrl) {
  if (ctrl->status) return;
  if (only_if_wide && !ctrl->wide) return;
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
  // The group keeps 2 * GW consecutive prefix sums of the low-priority queue in registers (win0: entries
  // wb .. wb+GW-1, win1: the next GW), with wb <= p < wb + GW, so that most gaps are searched without
  // touching memory.
  uint64_t wb = 0;
  int64_t win0 = INT64_MAX, win1 = INT64_MAX;
  if (WINDOW) {
    win0 = gl < L ? pe[l0 + gl] : INT64_MAX;
    win1 = GW + gl < L ? pe[l0 + GW + gl] : INT64_MAX;
  }

  // The predicted gaps of the next round are read while this round is worked on; without the window the prefix
  // sum at the head of the queue is read again only when the head has moved.
  int64_t next_g = gl < n_gaps ? pg[h0 + gl] : 0;
  int64_t head_pe = (!WINDOW && L > 0) ? pe[l0] : INT64_MAX;
  for (uint64_t i0 = 0; i0 < n_gaps; i0 += GW) {
    const uint64_t mine = i0 + gl;
    const int64_t my_g = next_g;
    next_g = mine + GW < n_gaps ? pg[h0 + mine + GW] : 0;
    uint32_t my_c = 0;
    int64_t my_f = 0;
    const uint32_t steps = static_cast<uint32_t>(n_gaps - i0 < GW ? n_gaps - i0 : GW);
    uint32_t k = 0;
    while (k < steps) {
      // Gaps that the head of the queue does not fit into take nothing and change nothing: every lane tests
      // its own gap against the head, and the group goes straight to the first gap that takes something.
      // (with the window the prefix sum at the head comes from the lane that holds entry p: wb <= p < wb + GW)
      const int64_t head_abs = WINDOW ? group_value<GW>(win0, gbase, static_cast<uint32_t>(p - wb))
                                      : head_pe;
      const int64_t head = p < L ? head_abs - consumed : INT64_MAX;
      const bool takes = gl >= k && gl < steps && my_g >= min_gap && my_g >= margin && head <= my_g - margin;
      const uint64_t tb = (ballot(takes) >> gbase) & gmask;
      if (tb == 0) break;
      k = static_cast<uint32_t>(__builtin_ctzll(tb));
      const int64_t G = group_value<GW>(my_g, gbase, k);
      uint32_t c = 0;
      int64_t f = 0;
      if (G >= min_gap && G >= margin && p < L) {
        const int64_t limit = consumed + (G - margin);
        int64_t last_fit = consumed;
        for (;;) {
          // candidate of this lane: queue entry p + c + gl, which lives in the window at idx
          int64_t val;
          if (WINDOW) {
            const uint32_t idx = static_cast<uint32_t>(p + c - wb) + gl;          // 0 .. 2 * GW - 2
            const int64_t a0 = static_cast<int64_t>(shfl_u64(static_cast<uint64_t>(win0), gbase + (idx & (GW - 1))));
            const int64_t a1 = static_cast<int64_t>(shfl_u64(static_cast<uint64_t>(win1), gbase + (idx & (GW - 1))));
            val = idx < GW ? a0 : a1;    // INT64_MAX beyond the end of the queue
          } else {
            const uint64_t j = p + c + gl;
            val = j < L ? pe[l0 + j] : INT64_MAX;
          }
          const bool fits = val <= limit;
          const uint64_t b = (ballot(fits) >> gbase) & gmask;
          const uint32_t cnt = (b == gmask) ? GW : static_cast<uint32_t>(__builtin_ctzll(~b));
          if (cnt > 0) last_fit = group_value<GW>(val, gbase, cnt - 1);
          c += cnt;
          // keep the window under the search position
          if (WINDOW && p + c >= wb + GW) {
            wb += GW;
            win0 = win1;
            win1 = wb + GW + gl < L ? pe[l0 + wb + GW + gl] : INT64_MAX;
          }
          if (cnt < GW) break;
        }
        f = last_fit - consumed;
        consumed = last_fit;
        p += c;
        if (!WINDOW && c > 0) head_pe = p < L ? pe[l0 + p] : INT64_MAX;
        if (p == L && c > 0 && !done) {
          completion = open[h0 + i0 + k] + f;
          done = true;
        }
      }
      if (gl == k) { my_c = c; my_f = f; }
      ++k;
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

// ---------------------------------------------------------------------------------------------
// One lane per scenario.
//
// When there are many scenarios, the cheapest way to run Algorithm 1 is its literal form, one lane per
// scenario: keep what is left of the current gap, and issue the head of the low-priority queue while
// its predicted duration fits.  A lane needs the predicted execution time of every low-priority
// launch once, in order, and the predicted (execution time, idle time) of every high-priority launch
// once, in order: two streams per lane.  They are stored as 32-bit numbers (4 and 8 bytes per launch
// instead of three 8-byte arrays); a prediction that does not fit 32 bits sets Ctrl::wide and the
// call is redone with the 64-bit kernels above.
//
// Each lane steps through its own scenario: a sub-step either opens the next gap or tries the next
// queue entry, so lanes of a wave do not wait for the slowest gap.  Streams are read 64 bytes per lane
// at a time into registers and parked in per-lane LDS rings one period later, which hides the memory
// latency; a lane whose ring is empty simply idles for a sub-step.  Results are staged
// in LDS and written 8 gaps at a time.  With one wave per SIMD (65,536 scenarios fill the chip exactly
// once) a SIMD issues one instruction of its wave every four cycles at best, so the kernel's time is its
// number of instructions: the tries after an opening read all their queue entries at once and ahead of
// use, and whatever can be derived when a gap's result is staged (its count, its filled time, its opening
// time) is not carried through the tries.

constexpr uint32_t WIDE32 = 0xffffffffu;   // 32-bit predictions must be below this

// Predicted values of every launch of the tasks that take part, in 32 bits:
//   lp_e[i]  execution time, for tasks used as low-priority queue; lp_total[t] their sum
//   hp_eg[i] (execution time, idle time), for tasks used as high-priority trace
// For the replay against actual idle times (actual != nullptr) the first word of hp_eg[i] holds the idle
// time that really followed launch i instead (clamped to WIDE32, which no filled time can reach).
// pred_done (may be null): tasks whose predictions exist already and are left alone.
__global__ void __launch_bounds__(PRED_THREADS)
k_gf_predict32(const uint64_t* __restrict__ ids, const uint64_t* __restrict__ off, uint32_t n_tasks,
               const fikit_row* __restrict__ rows, const uint64_t* __restrict__ row_off, const uint32_t* __restrict__ role,
               const uint32_t* __restrict__ lists, const int64_t* __restrict__ actual, uint32_t* __restrict__ lp_e,
               uint2* __restrict__ hp_eg, uint64_t* __restrict__ lp_total, uint32_t predictor,
               const uint32_t* __restrict__ pred_done, Ctrl* ctrl) {
  __shared__ PredTable tb;
  __shared__ uint64_t wave_tot[PRED_THREADS / WAVE];
  if (ctrl->status & (ERR_OFFSETS | ERR_TASK_INDEX | ERR_GAP_OFFSETS)) return;
  const uint32_t n_short = ctrl->n_class[0], n_longer = ctrl->n_class[1];   // final: set by an earlier kernel
  if (blockIdx.x >= n_short + n_longer) return;
  const uint32_t t = blockIdx.x < n_short ? lists[blockIdx.x] : lists[static_cast<uint64_t>(n_tasks) + (blockIdx.x - n_short)];
  const uint32_t rl = role[t];
  if (rl == 0) return;
  if (pred_done && pred_done[t]) return;   // (the profile kernels wrote this task's predictions already)
  const uint64_t base = off[t], len = off[t + 1] - base;
  const uint64_t r0 = row_off[t], nr = row_off[t + 1] - r0;
  const uint32_t tid = threadIdx.x;
  const bool in_lds = nr <= PRED_ROWS && (nr == 0 || rows[r0 + nr - 1].kernel_id != ~0ull);
  if (in_lds) {
    for (uint32_t h = tid; h < PRED_HT; h += PRED_THREADS) tb.key[h] = ~0ull;
    __syncthreads();
    for (uint32_t r = tid; r < nr; r += PRED_THREADS) {
      const fikit_row* row = rows + r0 + r;
      const uint64_t id = row->kernel_id;
      uint32_t h = (static_cast<uint32_t>(id >> 32) ^ static_cast<uint32_t>(id)) & (PRED_HT - 1);
      for (;;) {   // IDs of a task are distinct and fill at most half the table: a free slot exists
        const uint64_t old = atomicCAS(reinterpret_cast<unsigned long long*>(&tb.key[h]), ~0ull, id);
        if (old == ~0ull) break;
        h = (h + 1) & (PRED_HT - 1);
      }
      tb.e[h] = predicted_of(row->exec, predictor);
      tb.g[h] = predicted_of(row->gap, predictor);
    }
  }
  __syncthreads();
  bool unknown = false, wide = false, bad_actual = false;
  uint64_t total = 0;
  const bool even = ((base & 1) == 0);   // 16-byte accesses to the workspace arrays need an even first index
  const bool ids_vec = (reinterpret_cast<uintptr_t>(ids + base) & 15) == 0;   // and those to the caller's IDs an aligned address
  for (uint64_t i0 = 2 * static_cast<uint64_t>(tid); i0 < len; i0 += 2 * PRED_THREADS) {
    uint64_t id0 = 0, id1 = 0;
    const bool two = i0 + 1 < len;
    if (ids_vec && two) {
      const ulonglong2 v = *reinterpret_cast<const ulonglong2*>(ids + base + i0);
      id0 = v.x; id1 = v.y;
    } else {
      id0 = ids[base + i0];
      if (two) id1 = ids[base + i0 + 1];
    }
    int64_t e0 = 0, g0 = 0, e1 = 0, g1 = 0;
    unknown |= !predict_one(id0, in_lds, tb, rows, r0, nr, predictor, e0, g0);
    if (two) unknown |= !predict_one(id1, in_lds, tb, rows, r0, nr, predictor, e1, g1);
    wide |= static_cast<uint64_t>(e0) >= WIDE32 || static_cast<uint64_t>(g0) >= WIDE32 || static_cast<uint64_t>(e1) >= WIDE32 ||
            static_cast<uint64_t>(g1) >= WIDE32;
    const uint32_t a0 = static_cast<uint32_t>(e0), b0 = static_cast<uint32_t>(g0), a1 = static_cast<uint32_t>(e1),
                   b1 = static_cast<uint32_t>(g1);
    total += static_cast<uint64_t>(a0) + a1;
    uint32_t h0w = a0, h1w = a1;   // first word of the high-priority entries
    if (actual && (rl & ROLE_HP)) {
      // (the task's last launch has no idle time after it and its entry is never used as a gap)
      const int64_t x0 = i0 + 1 < len ? actual[base + i0] : 0, x1 = i0 + 2 < len ? actual[base + i0 + 1] : 0;
      bad_actual |= x0 < 0 || x1 < 0;
      h0w = static_cast<uint64_t>(x0) >= WIDE32 ? WIDE32 : static_cast<uint32_t>(x0);
      h1w = static_cast<uint64_t>(x1) >= WIDE32 ? WIDE32 : static_cast<uint32_t>(x1);
    }
    if (even && two) {
      if (rl & ROLE_LP) *reinterpret_cast<uint2*>(lp_e + base + i0) = make_uint2(a0, a1);
      if (rl & ROLE_HP) *reinterpret_cast<uint4*>(hp_eg + base + i0) = make_uint4(h0w, b0, h1w, b1);
    } else {
      if (rl & ROLE_LP) { lp_e[base + i0] = a0; if (two) lp_e[base + i0 + 1] = a1; }
      if (rl & ROLE_HP) { hp_eg[base + i0] = make_uint2(h0w, b0); if (two) hp_eg[base + i0 + 1] = make_uint2(h1w, b1); }
    }
  }
  total = wave_sum_u64(total);
  if (lane_id() == 0) wave_tot[tid >> 6] = total;
  __syncthreads();
  if (tid == 0) {
    uint64_t sum = 0;
    for (int w = 0; w < PRED_THREADS / WAVE; ++w) sum += wave_tot[w];
    lp_total[t] = sum;
  }
  if (unknown) atomicOr(&ctrl->status, ERR_UNKNOWN_ID);
  if (bad_actual) atomicOr(&ctrl->status, ERR_ACTUAL_GAP);
  if (wide) atomicOr(&ctrl->wide, 1u);
}

// The replay for predictions that do not fit 32 bits (Ctrl::wide): one lane per scenario steps through
// its gaps literally, on the 64-bit arrays of k_gf_predict (a low-priority kernel's predicted duration is the
// difference of two prefix sums).  Rare and slow on purpose; results are those of the 32-bit kernels.
__global__ void __launch_bounds__(256)
k_gf_replay_wide(const uint64_t* __restrict__ off, const uint32_t* __restrict__ hp_task, const uint32_t* __restrict__ lp_task,
                 uint64_t n_scen, const uint64_t* __restrict__ gap_off, const int64_t* __restrict__ pe,
                 const int64_t* __restrict__ pg, const int64_t* __restrict__ actual, int64_t margin, int64_t min_gap,
                 uint32_t feedback, uint32_t* __restrict__ fill_count, int64_t* __restrict__ filled_ns,
                 int64_t* __restrict__ delay_out, uint64_t* __restrict__ placed_out, Ctrl* ctrl) {
  if ((ctrl->status & ~ERR_ACTUAL_GAP) || !ctrl->wide) return;   // (the one bit this kernel itself may set)
  const uint64_t s = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (s >= n_scen) return;
  const uint32_t hp = hp_task[s], lp = lp_task[s];
  const uint64_t h0 = off[hp], H = off[hp + 1] - h0;
  const uint64_t l0 = off[lp], L = off[lp + 1] - l0;
  const uint64_t g0 = gap_off[s];
  uint64_t p = 0;
  int64_t consumed = 0, delay = 0;
  bool bad_actual = false;
  for (uint64_t i = 0; i + 1 < H; ++i) {
    const int64_t G = pg[h0 + i], a = actual[h0 + i];
    bad_actual |= a < 0;
    uint32_t c = 0;
    int64_t f = 0;
    if (G >= min_gap && G >= margin) {
      int64_t rem = G - margin;
      while (p < L) {
        const int64_t d = pe[l0 + p] - consumed;
        if (d > rem || (feedback && f >= a)) break;
        rem -= d; f += d; consumed += d;
        ++p; ++c;
      }
      if (f > a) delay += f - a;
    }
    fill_count[g0 + i] = c;
    filled_ns[g0 + i] = f;
  }
  if (bad_actual) atomicOr(&ctrl->status, ERR_ACTUAL_GAP);
  delay_out[s] = delay;
  placed_out[s] = p;
}

constexpr int LW_THREADS = 256;
constexpr uint32_t LW_OPENS = 4, LW_TRIES = 4;     // per period (between two rounds of stream reads / result writes):
                                                   // gaps opened, and queue entries tried per gap opened
constexpr uint32_t LW_LP_CHUNK = 16, LW_LP_CAP = 32;   // low-priority ring: entries read at a time, capacity
constexpr uint32_t LW_HP_CHUNK = 8, LW_HP_CAP = 16;    // high-priority ring
constexpr uint32_t LW_OUT_CHUNK = 8, LW_OUT_CAP = 32;  // staged results
// The first rows of the low-priority ring are kept a second time behind its last row, so that the LW_TRIES entries
// from any position on are consecutive rows (one address, constant offsets).
constexpr uint32_t LW_LP_MIRROR = LW_TRIES - 1;
static_assert(LW_LP_MIRROR < LW_LP_CHUNK, "the rows that are mirrored land together");

struct LaneWalkSmem {   // [entry][lane]: a lane's entries fall on one bank whatever position it is at
  uint32_t lp[LW_LP_CAP + LW_LP_MIRROR][LW_THREADS];
  uint32_t hp_e[LW_HP_CAP][LW_THREADS];
  uint32_t hp_g[LW_HP_CAP][LW_THREADS];
  uint32_t out_c[LW_OUT_CAP][LW_THREADS];
  uint32_t out_f[LW_OUT_CAP][LW_THREADS];
};

// Writes the staged results of gaps [first, first + count) (global gap numbers) of the calling lane.
__device__ __forceinline__ void lw_store_scalar(const LaneWalkSmem& sm, uint32_t tid, uint32_t first, uint32_t count,
                                                uint32_t* __restrict__ fill_count, int64_t* __restrict__ filled_ns) {
  for (uint32_t k = 0; k < count; ++k) {
    const uint32_t at = first + k;
    fill_count[at] = sm.out_c[at & (LW_OUT_CAP - 1)][tid];
    filled_ns[at] = static_cast<int64_t>(sm.out_f[at & (LW_OUT_CAP - 1)][tid]);
  }
}

// MODE 0: the plan on predictions (fill counts, filled time, completion time of the low-priority task).
// MODE 1 / 2: the same decisions replayed against the idle times that occurred, without / with real-time
// feedback (the runtime-feedback paragraph of the paper's scheduling section): the first word of a
// high-priority entry is then the actual idle time; with feedback nothing more is issued into a gap once
// the time filled has reached it; what runs past it delays the high-priority task, and the sum of these
// delays is written in place of the completion time.
enum : int { LW_PLAN = 0, LW_REPLAY = 1, LW_REPLAY_FEEDBACK = 2 };

template <int MODE>
__global__ void __launch_bounds__(LW_THREADS)
k_gf_walk_lanes(const uint64_t* __restrict__ off, const uint32_t* __restrict__ hp_task, const uint32_t* __restrict__ lp_task,
                uint64_t n_scen, const uint64_t* __restrict__ gap_off, const uint32_t* __restrict__ lp_e,
                const uint2* __restrict__ hp_eg, const uint64_t* __restrict__ lp_total, int64_t margin, int64_t min_gap,
                uint32_t* __restrict__ fill_count, int64_t* __restrict__ filled_ns, int64_t* __restrict__ completion_out,
                uint64_t* __restrict__ placed_out, uint32_t vec_ok, const Ctrl* ctrl) {
  extern __shared__ __align__(16) unsigned char lw_raw[];
  LaneWalkSmem& sm = *reinterpret_cast<LaneWalkSmem*>(lw_raw);
  if (ctrl->status || ctrl->wide) return;
  const uint32_t tid = threadIdx.x;
  const uint64_t s = static_cast<uint64_t>(blockIdx.x) * LW_THREADS + tid;
  const bool valid = s < n_scen;

  // positions are global element numbers (all below 2^32)
  uint32_t h0 = 0, hp_end = 0, l0 = 0, lp_end = 0, g_first = 0, n_gaps = 0;
  uint64_t total_lp = 0;
  if (valid) {
    const uint32_t hp = hp_task[s], lp = lp_task[s];
    h0 = static_cast<uint32_t>(off[hp]); hp_end = static_cast<uint32_t>(off[hp + 1]);
    l0 = static_cast<uint32_t>(off[lp]); lp_end = static_cast<uint32_t>(off[lp + 1]);
    g_first = static_cast<uint32_t>(gap_off[s]);
    n_gaps = hp_end > h0 ? hp_end - h0 - 1 : 0;
    total_lp = (MODE == LW_PLAN && lp_end > l0) ? lp_total[lp] : 0;
  }
  uint32_t hp_pos = h0, lp_pos = l0;                    // next entry of either stream
  uint32_t hp_landed = h0 & ~(LW_HP_CHUNK - 1), lp_landed = l0 & ~(LW_LP_CHUNK - 1);   // ring holds entries below these
  uint32_t hp_req = 0, lp_req = 0;
  bool hp_fly = false, lp_fly = false;
  uint4 hr[4], lr[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) hr[k] = lr[k] = make_uint4(0, 0, 0, 0);

  uint32_t g = g_first;              // global number of the next gap to report
  uint32_t flushed = g_first;        // results below this are in memory
  const uint32_t g_end = g_first + n_gaps;
  int64_t t_open = 0;                // predicted time line of the high-priority task
  uint32_t g_cur = 0;                // idle time of the gap opened last (its opening time is t_open - g_cur)
  int64_t completion;
  uint64_t consumed = 0;
  uint32_t rem = 0, rem_open = 0;    // what is left of the open gap's budget; the budget it opened with
  uint32_t lp_open = l0;             // position in the queue when the gap opened
  uint32_t ga = 0;                   // replay: the idle time that occurred after the launch whose gap is open
  int64_t delay = 0;                 // replay: by how much issued kernels ran past the gaps so far
  // a gap is used if it is at least min_gap and at least the margin long (32-bit idle times are below WIDE32)
  const int64_t floor64 = min_gap > margin ? min_gap : margin;
  const uint32_t gap_floor = floor64 >= static_cast<int64_t>(WIDE32) ? WIDE32 : static_cast<uint32_t>(floor64);
  const uint32_t margin32 = margin >= static_cast<int64_t>(WIDE32) ? WIDE32 : static_cast<uint32_t>(margin);
  bool in_gap = false;
  bool pending = false;               // a gap has closed and its result (c, f) is not staged yet
  bool finished = !valid || lp_end == l0;  // nothing left to step through (remaining gaps, if any, get zeros)

  for (;;) {
    // ---- once per period: park what was read, read on, write complete groups of results ----
    if (hp_fly) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t at = (hp_req + 2 * k) & (LW_HP_CAP - 1);
        sm.hp_e[at][tid] = hr[k].x; sm.hp_g[at][tid] = hr[k].y;
        sm.hp_e[at + 1][tid] = hr[k].z; sm.hp_g[at + 1][tid] = hr[k].w;
      }
      hp_landed = hp_req + LW_HP_CHUNK;
      hp_fly = false;
    }
    if (lp_fly) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t at = (lp_req + 4 * k) & (LW_LP_CAP - 1);
        const uint32_t v[4] = {lr[k].x, lr[k].y, lr[k].z, lr[k].w};
#pragma unroll
        for (uint32_t i = 0; i < 4; ++i) {
          sm.lp[at + i][tid] = v[i];
          if (at + i < LW_LP_MIRROR) sm.lp[LW_LP_CAP + at + i][tid] = v[i];
        }
      }
      lp_landed = lp_req + LW_LP_CHUNK;
      lp_fly = false;
    }
    if (!finished && hp_landed < hp_end && static_cast<int32_t>(hp_landed - hp_pos) <= static_cast<int32_t>(LW_HP_CAP - LW_HP_CHUNK)) {
      const uint4* src = reinterpret_cast<const uint4*>(hp_eg + hp_landed);
#pragma unroll
      for (int k = 0; k < 4; ++k) hr[k] = src[k];
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
      lw_store_scalar(sm, tid, flushed, cnt, fill_count, filled_ns);
      flushed += cnt;
    }
    while (flushed + LW_OUT_CHUNK <= g) {
      if (vec_ok) {
        const uint32_t at = flushed & (LW_OUT_CAP - 1);
        uint32_t cc[LW_OUT_CHUNK], ff[LW_OUT_CHUNK];
#pragma unroll
        for (uint32_t k = 0; k < LW_OUT_CHUNK; ++k) { cc[k] = sm.out_c[at + k][tid]; ff[k] = sm.out_f[at + k][tid]; }
        uint4* oc = reinterpret_cast<uint4*>(fill_count + flushed);
        oc[0] = make_uint4(cc[0], cc[1], cc[2], cc[3]);
        oc[1] = make_uint4(cc[4], cc[5], cc[6], cc[7]);
        uint4* of = reinterpret_cast<uint4*>(filled_ns + flushed);
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) of[k] = make_uint4(ff[2 * k], 0u, ff[2 * k + 1], 0u);
      } else {
        lw_store_scalar(sm, tid, flushed, LW_OUT_CHUNK, fill_count, filled_ns);
      }
      flushed += LW_OUT_CHUNK;
    }
    if (__all(finished)) break;

    // ---- one period: LW_OPENS times { stage the result of the gap that closed, take the next
    // high-priority launch and open its gap; LW_TRIES times try the head of the queue }.  Written
    // without branches; a lane whose ring is empty, or whose gap is still open when a new one could be
    // taken, simply idles in that sub-step. ----
    const uint32_t lp_lim = lp_landed < lp_end ? lp_landed : lp_end;   // tries look at entries below this
#pragma unroll
    for (uint32_t o = 0; o < LW_OPENS; ++o) {
      // the queue entries that the tries after this opening may look at, read ahead of the opening's own work
      uint32_t w[LW_TRIES];
#pragma unroll
      for (uint32_t k = 0; k < LW_TRIES; ++k) w[k] = sm.lp[(lp_pos & (LW_LP_CAP - 1)) + k][tid];
      {
        // the whole queue has been issued (noticed here, not in the tries): the open gap is its last, the time line and f
        // stay as they are from here on
        const bool emptied = in_gap && lp_pos == lp_end;
        pending = pending || emptied;
        in_gap = in_gap && !emptied;
        finished = finished || emptied;
        // what the gap that is open, or has just closed, took (the tries only move lp_pos and rem; a gap that was
        // skipped took nothing)
        const uint32_t c = lp_pos - lp_open, f = rem_open - rem;
        // (a staging slot that is written early is simply written again)
        sm.out_c[g & (LW_OUT_CAP - 1)][tid] = c;
        sm.out_f[g & (LW_OUT_CAP - 1)][tid] = f;
        g += pending ? 1u : 0u;
        consumed += pending ? f : 0u;
        if (MODE != LW_PLAN) delay += (pending && f > ga) ? static_cast<int64_t>(f - ga) : 0;
        const uint32_t E = sm.hp_e[hp_pos & (LW_HP_CAP - 1)][tid], G = sm.hp_g[hp_pos & (LW_HP_CAP - 1)][tid];
        // between gaps: the next high-priority launch runs, then its gap opens (the last launch has none)
        const bool idle = !finished && !in_gap;
        const bool at_end = idle && hp_pos == hp_end;
        const bool take = idle && !at_end && hp_pos < hp_landed;
        hp_pos += take ? 1u : 0u;
        const bool last = take && hp_pos == hp_end;
        const bool gap = take && !last;
        if (MODE == LW_PLAN) {
          t_open += take ? static_cast<int64_t>(E) : 0;
          t_open += gap ? static_cast<int64_t>(G) : 0;     // (the time line after the gap: the gap opened g_cur earlier)
          g_cur = gap ? G : g_cur;
        }
        const bool usable = gap && G >= gap_floor;
        if (MODE != LW_PLAN) ga = usable ? E : ga;
        in_gap = in_gap || usable;
        // a gap that is skipped is closed at once and reports zeros when the next one is opened
        pending = gap && !usable;
        rem = gap ? G - margin32 : rem;
        rem_open = gap ? rem : rem_open;
        lp_open = gap ? lp_pos : lp_open;
        finished = finished || at_end || last;
      }
      // In a gap: does the head of the queue fit into what is left?  Then the entry behind it, and so on: an entry is
      // tried only behind one that fit, so the k-th try of an opening looks at the k-th entry from where the queue stood,
      // and the tries end at the first entry that does not fit.  The running sums of those entries only grow (a sum
      // beyond 32 bits stays at the largest value, which no gap reaches), so the number of entries that fit is the
      // number of running sums within what is left, at most the entries that have landed.
      const int32_t room = static_cast<int32_t>(lp_lim - lp_pos);   // entries that have landed (<= 0: none)
      uint32_t run[LW_TRIES];
      run[0] = w[0];
#pragma unroll
      for (uint32_t k = 1; k < LW_TRIES; ++k) run[k] = __builtin_elementwise_add_sat(run[k - 1], w[k]);
      uint32_t n = 0;
#pragma unroll
      for (uint32_t k = 0; k < LW_TRIES; ++k) n += run[k] <= rem ? 1u : 0u;
      if (MODE == LW_REPLAY_FEEDBACK) {
        // (with feedback: the next high-priority request has arrived once the time filled reaches the actual gap;
        // an entry is issued only while the time filled before it is below that)
        const uint32_t f0 = rem_open - rem;
        uint32_t n2 = f0 < ga ? 1u : 0u;
#pragma unroll
        for (uint32_t k = 1; k < LW_TRIES; ++k) n2 += __builtin_elementwise_add_sat(f0, run[k - 1]) < ga ? 1u : 0u;
        n = n < n2 ? n : n2;
      }
      const int32_t capped = room < static_cast<int32_t>(LW_TRIES) ? room : static_cast<int32_t>(LW_TRIES);
      const uint32_t avail = capped > 0 ? static_cast<uint32_t>(capped) : 0u;
      const uint32_t nfit = in_gap ? (n < avail ? n : avail) : 0u;
      const bool close = in_gap && n < avail;   // an entry that was there did not fit: the gap is closed
      uint32_t taken = 0;
#pragma unroll
      for (uint32_t k = 0; k < LW_TRIES; ++k) taken = nfit > k ? run[k] : taken;
      rem -= taken;
      pending = pending || close;
      in_gap = in_gap && !close;
      lp_pos += nfit;
    }
  }

  if (!valid) return;
  const uint32_t c = lp_pos - lp_open, f = rem_open - rem;   // of the last gap that was opened
  if (pending) {
    sm.out_c[g & (LW_OUT_CAP - 1)][tid] = c;
    sm.out_f[g & (LW_OUT_CAP - 1)][tid] = f;
    ++g;
    consumed += f;
    if (MODE != LW_PLAN && f > ga) delay += static_cast<int64_t>(f - ga);
  }
  // what is still staged, then zeros for the gaps after the queue ran empty
  lw_store_scalar(sm, tid, flushed, g - flushed, fill_count, filled_ns);
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
  // the whole queue has been issued: the last of it into the gap opened last, after which the time line stood still
  const bool done = lp_pos == lp_end;
  completion = done ? t_open - static_cast<int64_t>(g_cur) + static_cast<int64_t>(f) : t_open + static_cast<int64_t>(total_lp - consumed);
  completion_out[s] = MODE == LW_PLAN ? completion : delay;
  placed_out[s] = lp_pos - l0;
}


}  // namespace fikit
