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

// Sorts tasks into work lists by length: lists[c * n_tasks ...] for c = 0 (up to len_small launches),
// 1 (up to len_mid), 2 (up to len_max); longer tasks start on the long-task path (gflag 1).  A kernel
// that handles one class is launched over that class's list, so that every workgroup it starts has
// work of similar size (workgroups are handed to compute units in turn: a launch in which busy and
// idle workgroups alternate would keep only some of the units busy).  Order inside a list is arbitrary.
__global__ void k_classify(const uint64_t* __restrict__ off, uint32_t n_tasks, uint32_t len_small, uint32_t len_mid,
                           uint32_t len_max, uint32_t* __restrict__ gflag, uint32_t* __restrict__ dcount,
                           uint32_t* __restrict__ lists, Ctrl* ctrl) {
  if (ctrl->status & ERR_OFFSETS) return;
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  uint32_t c = 3;   // 0, 1, 2: work list; 3: none
  bool is_long = false;
  if (t <= n_tasks) dcount[t] = 0;
  if (t < n_tasks) {
    const uint64_t len = off[t + 1] - off[t];
    is_long = len > len_max;
    gflag[t] = is_long ? 1u : 0u;
    if (!is_long && len > 0) c = len <= len_small ? 0u : (len <= len_mid ? 1u : 2u);
  }
  for (uint32_t k = 0; k < 3; ++k) {
    const uint32_t pos = wave_append(&ctrl->n_class[k], c == k);
    if (c == k) lists[static_cast<uint64_t>(k) * n_tasks + pos] = static_cast<uint32_t>(t);
  }
  const uint64_t longs = ballot(is_long);
  if (longs && lane_id() == 0) {
    atomicAdd(reinterpret_cast<unsigned long long*>(&ctrl->n_general), static_cast<unsigned long long>(__popcll(longs)));
    atomicAdd(reinterpret_cast<unsigned long long*>(&ctrl->n_long), static_cast<unsigned long long>(__popcll(longs)));
  }
}

// Execution time and idle time of every launch as they stand in the trace (Section 3.2, "Measuring the
// execution and idle time of kernel"); task boundaries are put right by k_measure_task_ends afterwards.
__global__ void __launch_bounds__(256)
k_measure(const fikit_launch* __restrict__ rec, uint64_t n, int64_t* __restrict__ exec_ns, int64_t* __restrict__ gap_ns,
          Ctrl* ctrl) {
  if (ctrl->status & ERR_OFFSETS) return;
  const uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int64_t start = rec[i].start_ns, end = rec[i].end_ns;
  if (end < start) atomicOr(&ctrl->status, ERR_BAD_RECORD);
  exec_ns[i] = end - start;
  int64_t g = GAP_NONE;
  if (i + 1 < n && rec[i + 1].run == rec[i].run) { g = rec[i + 1].start_ns - end; g = g < 0 ? 0 : g; }   // (same run)
  gap_ns[i] = g;
}

// The last launch of every task has no idle time after it (whatever run the next task's first launch names).
__global__ void k_measure_task_ends(const uint64_t* __restrict__ off, uint32_t n_tasks, int64_t* __restrict__ gap_ns,
                                    const Ctrl* ctrl) {
  if (ctrl->status & ERR_OFFSETS) return;
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (t < n_tasks && off[t + 1] > off[t]) gap_ns[off[t + 1] - 1] = GAP_NONE;
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

}  // namespace fikit
