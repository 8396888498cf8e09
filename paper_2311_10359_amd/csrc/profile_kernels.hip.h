// Kernel ID hashing and per-launch measurement (Section 3.2, "Identifying each kernel" and
// "Measuring the execution and idle time of kernel"), plus small bookkeeping kernels.
#pragma once

#include "common.hip.h"

namespace fikit {

__global__ void k_clear_ctrl(Ctrl* ctrl) {
  if (threadIdx.x < sizeof(Ctrl) / 4) reinterpret_cast<uint32_t*>(ctrl)[threadIdx.x] = 0;
}

// Fills `count` 32-bit words with `value` (used instead of memset so that a caller may capture
// the stream into a graph).
__global__ void k_fill_u32(uint32_t* __restrict__ p, uint64_t count, uint32_t value) {
  uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
  for (; i < count; i += stride) p[i] = value;
}

// Checks the CSR task offsets: first 0, non-decreasing, last == n.
__global__ void k_validate_offsets(const uint64_t* __restrict__ off, uint32_t n_tasks, uint64_t n, Ctrl* ctrl) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  bool bad = false;
  if (t < n_tasks) {
    const uint64_t a = off[t], b = off[t + 1];
    bad = (a > b) || (b > n);
    if (t == 0 && a != 0) bad = true;
    if (t == n_tasks - 1 && b != n) bad = true;
  } else if (t == 0 && n_tasks == 0) {
    bad = (off[0] != 0) || (n != 0);
  }
  if (bad) atomicOr(&ctrl->status, ERR_OFFSETS);
}

// Tasks longer than max_fused launches take the general sort-based path from the start.
__global__ void k_classify(const uint64_t* __restrict__ off, uint32_t n_tasks, uint32_t max_fused, uint32_t* __restrict__ gflag,
                           uint32_t* __restrict__ dcount, Ctrl* ctrl) {
  if (ctrl->status & ERR_OFFSETS) return;
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (t > n_tasks) return;
  dcount[t] = 0;
  if (t == n_tasks) return;
  const bool is_long = (off[t + 1] - off[t]) > max_fused;
  gflag[t] = is_long ? 1u : 0u;
  if (is_long) {
    atomicAdd(reinterpret_cast<unsigned long long*>(&ctrl->n_general), 1ull);
    atomicAdd(reinterpret_cast<unsigned long long*>(&ctrl->n_long), 1ull);
  }
}

// FNV-1a, 64 bit, over the eight little-endian 32-bit words that hold a launch's identity
// (name id, grid x y z, block x y z, dynamic shared-memory bytes): for each byte in memory
// order, xor it into the hash, then multiply by the FNV prime 2^40 + 0x1b3 modulo 2^64.
__device__ __forceinline__ uint64_t kernel_id_of(const uint32_t (&w)[8]) {
  uint32_t lo = 0x84222325u, hi = 0xcbf29ce4u;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      lo ^= (w[k] >> (8 * b)) & 0xffu;
      // (hi:lo) * (2^40 + 0x1b3): the 2^40 term only reaches the high word as lo << 8.
      const uint32_t hi_part = hi * 0x1b3u + (lo << 8);
      const uint64_t prod = static_cast<uint64_t>(lo) * 0x1b3u + (static_cast<uint64_t>(hi_part) << 32);
      lo = static_cast<uint32_t>(prod);
      hi = static_cast<uint32_t>(prod >> 32);
    }
  }
  return (static_cast<uint64_t>(hi) << 32) | lo;
}

// One launch record per thread: Kernel ID, execution time K = end - start, and the idle time
// G = max(0, start of the following record - end).  Whether the following record belongs to the
// same task is settled afterwards by k_mark_task_ends, which overwrites the G of every task's
// last launch with GAP_NONE.
constexpr int HASH_BLOCK = 256;
__global__ void __launch_bounds__(HASH_BLOCK)
k_hash_measure(const fikit_launch* __restrict__ rec, uint64_t n, uint64_t* __restrict__ ids,
               int64_t* __restrict__ exec_out, int64_t* __restrict__ gap_out, Ctrl* ctrl) {
  const uint64_t i = static_cast<uint64_t>(blockIdx.x) * HASH_BLOCK + threadIdx.x;
  if (i >= n) return;
  const uint4* p = reinterpret_cast<const uint4*>(rec + i);
  const uint4 a = p[0];
  const uint4 b = p[1];
  const uint4 c = p[2];  // start_ns, end_ns
  int64_t next_start = 0;
  const bool has_next = (i + 1 < n);
  if (has_next) next_start = rec[i + 1].start_ns;
  const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
  const uint64_t id = kernel_id_of(w);
  const int64_t start = static_cast<int64_t>((static_cast<uint64_t>(c.y) << 32) | c.x);
  const int64_t end = static_cast<int64_t>((static_cast<uint64_t>(c.w) << 32) | c.z);
  if (end < start) atomicOr(&ctrl->status, ERR_BAD_RECORD);
  int64_t gap = GAP_NONE;
  if (has_next) {
    gap = next_start - end;
    if (gap < 0) gap = 0;
  }
  ids[i] = id;
  exec_out[i] = end - start;
  gap_out[i] = gap;
}

// The last launch of every non-empty task has no idle time after it.
__global__ void k_mark_task_ends(const uint64_t* __restrict__ off, uint32_t n_tasks, int64_t* __restrict__ gap,
                                 const Ctrl* ctrl) {
  if (ctrl->status & ERR_OFFSETS) return;
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (t >= n_tasks) return;
  const uint64_t a = off[t], b = off[t + 1];
  if (b > a) gap[b - 1] = GAP_NONE;
}

}  // namespace fikit
