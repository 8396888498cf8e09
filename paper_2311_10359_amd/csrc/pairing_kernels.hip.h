// The best low-priority partner of every high-priority task among evaluated combinations (the paper's
// discussion section, "What Tasks are Suitable for Sharing a GPU").
#pragma once

#include "common.hip.h"

namespace fikit {

constexpr int PAIR_THREADS = 256;

// One workgroup per scenario: checks the scenario, sums the time filled in its gaps (8 B read per gap)
// and raises the largest filled time seen for its high-priority task.
__global__ void __launch_bounds__(PAIR_THREADS)
k_pair_sum(const uint32_t* __restrict__ hp_task, const uint32_t* __restrict__ lp_task, uint64_t n_scen, uint32_t n_tasks,
           const uint64_t* __restrict__ gap_off, uint64_t n_gaps, const int64_t* __restrict__ filled_ns,
           int64_t* __restrict__ scen_filled, long long* __restrict__ top_filled, Ctrl* ctrl) {
  __shared__ uint64_t part[PAIR_THREADS / WAVE];
  const uint64_t s = blockIdx.x;
  const uint32_t tid = threadIdx.x;
  const uint32_t hp = hp_task[s], lp = lp_task[s];
  const uint64_t g0 = gap_off[s], g1 = gap_off[s + 1];
  if (hp >= n_tasks || lp >= n_tasks) {
    if (tid == 0) atomicOr(&ctrl->status, ERR_TASK_INDEX);
    return;
  }
  if (g1 < g0 || g1 > n_gaps || (s == 0 && g0 != 0)) {
    if (tid == 0) atomicOr(&ctrl->status, ERR_GAP_OFFSETS);
    return;
  }
  uint64_t acc[4] = {0, 0, 0, 0};      // (sums wrap like the oracle's additions)
  uint64_t i = g0 + tid;
  for (; i + 3 * PAIR_THREADS < g1; i += 4 * PAIR_THREADS) {
#pragma unroll
    for (int k = 0; k < 4; ++k) acc[k] += static_cast<uint64_t>(filled_ns[i + k * PAIR_THREADS]);
  }
  for (; i < g1; i += PAIR_THREADS) acc[0] += static_cast<uint64_t>(filled_ns[i]);
  const uint64_t mine = wave_sum_u64(acc[0] + acc[1] + acc[2] + acc[3]);
  if (lane_id() == 0) part[tid >> 6] = mine;
  __syncthreads();
  if (tid == 0) {
    uint64_t total = 0;
#pragma unroll
    for (int w = 0; w < PAIR_THREADS / WAVE; ++w) total += part[w];
    scen_filled[s] = static_cast<int64_t>(total);
    atomicMax(&top_filled[hp], static_cast<long long>(total));
  }
}

// Among the scenarios of a task with the largest filled time: the earliest completion of the partner.
__global__ void k_pair_soonest(const uint32_t* __restrict__ hp_task, uint64_t n_scen, const int64_t* __restrict__ scen_filled,
                               const int64_t* __restrict__ completion, const long long* __restrict__ top_filled,
                               long long* __restrict__ soonest, const Ctrl* ctrl) {
  if (ctrl->status) return;
  const uint64_t s = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (s >= n_scen) return;
  const uint32_t hp = hp_task[s];
  if (scen_filled[s] == top_filled[hp]) atomicMin(&soonest[hp], static_cast<long long>(completion[s]));
}

// Among those: the first scenario.
__global__ void k_pair_first(const uint32_t* __restrict__ hp_task, uint64_t n_scen, const int64_t* __restrict__ scen_filled,
                             const int64_t* __restrict__ completion, const long long* __restrict__ top_filled,
                             const long long* __restrict__ soonest, unsigned long long* __restrict__ best_scenario,
                             const Ctrl* ctrl) {
  if (ctrl->status) return;
  const uint64_t s = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (s >= n_scen) return;
  const uint32_t hp = hp_task[s];
  if (scen_filled[s] == top_filled[hp] && completion[s] == soonest[hp]) atomicMin(&best_scenario[hp], static_cast<unsigned long long>(s));
}

// Start values per task (no memset: the stream may be under graph capture).
__global__ void k_pair_init(uint32_t n_tasks, long long* __restrict__ top_filled, long long* __restrict__ soonest,
                            unsigned long long* __restrict__ best_scenario) {
  const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_tasks) return;
  top_filled[t] = INT64_MIN;
  soonest[t] = INT64_MAX;
  best_scenario[t] = ~0ull;
}

// The partner and the filled time of the scenario that was picked; a task that heads no scenario gets
// the "none" values.
__global__ void k_pair_finish(uint32_t n_tasks, const uint32_t* __restrict__ lp_task, const unsigned long long* __restrict__ best_scenario,
                              uint32_t* __restrict__ best_lp, long long* __restrict__ top_filled, const Ctrl* ctrl) {
  if (ctrl->status) return;
  const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_tasks) return;
  const unsigned long long b = best_scenario[t];
  best_lp[t] = b == ~0ull ? ~0u : lp_task[b];
  if (b == ~0ull) top_filled[t] = 0;
}

}  // namespace fikit
