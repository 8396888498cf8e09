// Merging the profile of further runs into the profile of the runs so far (Section 3.2: the statistics
// run over all T measured runs of a task; a run of N kernels has N - 1 idle times, so profiles taken run
// by run and merged leave the idle time between runs out).
#pragma once

#include "common.hip.h"

namespace fikit {

constexpr int MERGE_THREADS = 256;
constexpr uint32_t MERGE_IDS = 3072;      // IDs of a task and input kept in LDS for the searches

struct MergeSmem {
  uint64_t ida[MERGE_IDS];
  uint64_t idb[MERGE_IDS];
  uint32_t aux[8];
  uint32_t partner[MERGE_THREADS];   // per row of the round: its row in the other table, or MERGE_NONE
  uint32_t place[MERGE_THREADS];     // where it goes in the task's output, or MERGE_NONE: nowhere
};
constexpr uint32_t MERGE_NONE = 0xffffffffu;

// Number of rows of `rows[0..n)` (ordered by ID) whose ID is below `id`; *found: one of them equals it.
// `ids` is the LDS copy of the IDs, or null.
__device__ __forceinline__ uint32_t ids_below(const fikit_row* __restrict__ rows, const uint64_t* ids, uint32_t n, uint64_t id,
                                              bool* found) {
  uint32_t lo = 0, hi = n;
  while (lo < hi) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    const uint64_t v = ids ? ids[mid] : rows[mid].kernel_id;
    if (v < id) lo = mid + 1; else hi = mid;
  }
  *found = lo < n && (ids ? ids[lo] : rows[lo].kernel_id) == id;
  return lo;
}

// One 8-byte field of a merged row.  f: the field's number in the row (0 ID, 1 task, 2..7 the execution
// times' count, sum, min, max, p50, p95, 8..13 the same of the idle times, 14..15 reserved); x, y: the field
// in the two rows; cx, cy: the sample counts of the field's block in the two rows.
__device__ __forceinline__ uint64_t merge_field(uint32_t f, uint64_t x, uint64_t y, uint64_t cx, uint64_t cy) {
  if (f < 2 || f >= 14) return x;
  if (cx == 0) return y;
  if (cy == 0) return x;
  const uint32_t kind = (f - 2) % 6;
  const int64_t sx = static_cast<int64_t>(x), sy = static_cast<int64_t>(y);
  if (kind <= 1) return x + y;                                            // count, sum (modulo 2^64)
  if (kind == 2) return static_cast<uint64_t>(sx < sy ? sx : sy);         // min
  if (kind == 3) return static_cast<uint64_t>(sx > sy ? sx : sy);         // max
  return cy > cx ? y : x;   // the percentiles of the union are not known: those of the input with more samples stand in
}

// Writes the planned rows of a round (sm.place / sm.partner, `rows` of them, taken from src[first ..]): sixteen
// lanes per row, one 8-byte field each, so that a wave reads and writes whole rows side by side.
__device__ __forceinline__ void merge_write_round(const MergeSmem& sm, const fikit_row* __restrict__ src, uint32_t first,
                                                  uint32_t rows, const fikit_row* __restrict__ other, fikit_row* __restrict__ out) {
  const uint32_t tid = threadIdx.x, f = tid & 15u;
  const int row_lane0 = static_cast<int>(lane_id() - f);
  for (uint32_t r = tid >> 4; r < rows; r += MERGE_THREADS / 16) {      // (the sixteen lanes of a row stay together)
    const uint32_t place = sm.place[r], partner = sm.partner[r];
    const uint64_t x = reinterpret_cast<const uint64_t*>(src + first + r)[f];
    const uint64_t y = partner != MERGE_NONE ? reinterpret_cast<const uint64_t*>(other + partner)[f] : 0;
    const int count_lane = row_lane0 + (f < 8 ? 2 : 8);
    const uint64_t cx = shfl_u64(x, count_lane), cy = shfl_u64(y, count_lane);
    const uint64_t v = partner != MERGE_NONE ? merge_field(f, x, y, cx, cy) : x;
    if (place != MERGE_NONE) reinterpret_cast<uint64_t*>(out + place)[f] = v;
  }
}

// MODE 0: checks both inputs of a task (task field, IDs strictly ascending) and counts the rows of the
// union into dcount[t].  MODE 1: writes the union's rows at row_off[t].. in ID order.
// One workgroup per task; rank of an ID in the union = IDs below it in a + IDs below it in b - IDs below
// it that are in both (a running count of the matched rows seen so far).
template <int MODE>
__global__ void __launch_bounds__(MERGE_THREADS)
k_merge(const fikit_row* __restrict__ a, const uint64_t* __restrict__ a_off, const fikit_row* __restrict__ b,
        const uint64_t* __restrict__ b_off, uint32_t n_tasks, uint32_t* __restrict__ dcount,
        const uint64_t* __restrict__ row_off, fikit_row* __restrict__ out, Ctrl* ctrl) {
  __shared__ MergeSmem sm;
  if (ctrl->status) return;    // (the offsets have been checked by now: with valid offsets every row read is in bounds)
  const uint32_t tid = threadIdx.x;
  for (uint32_t t = blockIdx.x; t < n_tasks; t += gridDim.x) {
    const uint64_t a0 = a_off[t], a1 = a_off[t + 1], b0 = b_off[t], b1 = b_off[t + 1];
    if (a1 < a0 || b1 < b0 || a1 - a0 >= (1ull << 32) || b1 - b0 >= (1ull << 32) || (t == 0 && (a0 != 0 || b0 != 0))) {
      if (tid == 0) { atomicOr(&ctrl->status, ERR_OFFSETS); if (MODE == 0) dcount[t] = 0; }
      continue;    // (the same for all threads)
    }
    const uint32_t na = static_cast<uint32_t>(a1 - a0), nb = static_cast<uint32_t>(b1 - b0);
    const fikit_row* ra = a + a0;
    const fikit_row* rb = b + b0;
    const bool in_lds = na <= MERGE_IDS && nb <= MERGE_IDS;
    __syncthreads();   // (the previous task's searches are over)
    if (in_lds) {
      for (uint32_t i = tid; i < na; i += MERGE_THREADS) sm.ida[i] = ra[i].kernel_id;
      for (uint32_t i = tid; i < nb; i += MERGE_THREADS) sm.idb[i] = rb[i].kernel_id;
    }
    __syncthreads();
    const uint64_t* ida = in_lds ? sm.ida : nullptr;
    const uint64_t* idb = in_lds ? sm.idb : nullptr;
    bool bad = false;
    uint32_t carry = 0;      // matched rows of a before this round
    for (uint32_t i0 = 0; i0 < na; i0 += MERGE_THREADS) {
      const uint32_t i = i0 + tid;
      bool found = false;
      uint32_t below = 0;
      uint64_t id = 0;
      if (i < na) {
        id = ida ? ida[i] : ra[i].kernel_id;
        below = ids_below(rb, idb, nb, id, &found);
        if (MODE == 0) bad |= ra[i].task != t || (i > 0 && (ida ? ida[i - 1] : ra[i - 1].kernel_id) >= id);
      }
      uint32_t total;
      const uint32_t before = block_excl_scan_256(found ? 1u : 0u, sm.aux, total);
      if (MODE == 1) {
        sm.partner[tid] = found ? below : MERGE_NONE;
        sm.place[tid] = i < na ? i + below - (carry + before) : MERGE_NONE;
        __syncthreads();
        merge_write_round(sm, ra, i0, na - i0 < MERGE_THREADS ? na - i0 : MERGE_THREADS, rb, out + row_off[t]);
        __syncthreads();
      }
      carry += total;
    }
    const uint32_t matched = carry;
    carry = 0;               // matched rows of b before this round
    for (uint32_t k0 = 0; k0 < nb; k0 += MERGE_THREADS) {
      const uint32_t k = k0 + tid;
      bool found = false;
      uint32_t below = 0;
      if (k < nb) {
        const uint64_t id = idb ? idb[k] : rb[k].kernel_id;
        if (MODE == 1) below = ids_below(ra, ida, na, id, &found);
        if (MODE == 0) bad |= rb[k].task != t || (k > 0 && (idb ? idb[k - 1] : rb[k - 1].kernel_id) >= id);
      }
      if (MODE == 1) {
        uint32_t total;
        const uint32_t before = block_excl_scan_256(found ? 1u : 0u, sm.aux, total);
        sm.partner[tid] = MERGE_NONE;
        sm.place[tid] = (k < nb && !found) ? k + below - (carry + before) : MERGE_NONE;    // (matched rows went out with a's)
        __syncthreads();
        merge_write_round(sm, rb, k0, nb - k0 < MERGE_THREADS ? nb - k0 : MERGE_THREADS, ra, out + row_off[t]);
        __syncthreads();
        carry += total;
      }
    }
    if (MODE == 0) {
      if (bad) atomicOr(&ctrl->status, ERR_ROWS);
      if (tid == 0) dcount[t] = na + nb - matched;
    }
  }
  if (MODE == 0 && blockIdx.x == 0 && tid == 0) dcount[n_tasks] = 0;   // (the scan leaves the total here)
}

}  // namespace fikit
