// Shared device helpers for the FIKIT kernels (gfx950, 64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fikit.h"

namespace fikit {

constexpr int WAVE = 64;

// Sentinel for "this launch is the last of its task and has no idle time after it".
// Real idle times are clamped to >= 0, so a negative value cannot be a sample.
constexpr int64_t GAP_NONE = -1;

// Sticky error bits collected on the device during a call.
enum : uint32_t {
  ERR_OFFSETS = 1u << 0,     // task offsets not monotone / wrong end
  ERR_BAD_RECORD = 1u << 1,  // end_ns < start_ns
  ERR_UNKNOWN_ID = 1u << 2,  // launch ID without a row in its task's profile
  ERR_TASK_INDEX = 1u << 3,  // scenario names a task >= n_tasks
  ERR_GAP_OFFSETS = 1u << 4, // scenario gap offsets do not match the trace lengths
  ERR_ACTUAL_GAP = 1u << 5,  // replay: negative actual idle time after a launch that has a gap
  ERR_LP_LIST = 1u << 6,     // priority queues: list offsets not monotone, or a level outside 1..9
  ERR_LP_LIMIT = 1u << 7,    // priority queues: more low-priority tasks or launches in a scenario than supported
  ERR_ROWS = 1u << 8,        // merge: a row in the wrong task, or IDs of a task not strictly ascending
  ERR_WAIT = 1u << 9,        // a tile of the sort gave up waiting for the tile before it (must not happen)
};

// What a task is used as by the scenarios of a gap-fill call.
constexpr uint32_t ROLE_HP = 1u, ROLE_LP = 2u;

// Control block at the start of the workspace; cleared by k_clear_ctrl at the start of a call.
struct Ctrl {
  uint32_t status;        // ERR_* bits
  uint32_t wide;          // gap fill: a prediction did not fit 32 bits, the 64-bit kernels take over;
                          // profile: the short sort left some task's keys out of order
  uint64_t n_big_tiles;   // tiles of the tasks sorted by the multi-pass path
  uint64_t n_rows;        // number of (task, ID) rows
  uint64_t n_general;     // tasks that take the general sort-based path
  uint64_t n_long;        // tasks too long for the one-workgroup path
  uint64_t n_heads;       // rows found by the general path
  uint32_t n_class[4];    // length of the work lists (small, mid, medium tasks or units); [3]: priority queues, the
                          // largest number of low-priority tasks of a scenario
};
static_assert(sizeof(Ctrl) == 64, "control block is 64 bytes");

__device__ __forceinline__ uint32_t lane_id() { return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }

// Number of set bits of a 64-bit wave mask in lanes below the calling lane.
__device__ __forceinline__ uint32_t popc_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

__device__ __forceinline__ uint64_t ballot(bool p) { return __ballot(p); }

template <typename T>
__device__ __forceinline__ T shfl(T v, int src) { return __shfl(v, src, WAVE); }

__device__ __forceinline__ uint64_t shfl_u64(uint64_t v, int src) {
  uint32_t lo = __shfl(static_cast<uint32_t>(v), src, WAVE);
  uint32_t hi = __shfl(static_cast<uint32_t>(v >> 32), src, WAVE);
  return (static_cast<uint64_t>(hi) << 32) | lo;
}

// The value that lane `src` holds, where `src` is the same in every lane of the wave: no trip through the LDS
// crossbar as for a shuffle, the lane is selected by a scalar.
__device__ __forceinline__ uint64_t read_lane_u64(uint64_t v, uint32_t src) {
  const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(static_cast<uint32_t>(v)), static_cast<int>(src)));
  const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(static_cast<uint32_t>(v >> 32)), static_cast<int>(src)));
  return (static_cast<uint64_t>(hi) << 32) | lo;
}

// A 16-byte load that tells the caches that its data will not be used again.
typedef uint32_t u32x4_native __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_once(const uint4* p) {
  const u32x4_native v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_native*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int m) {
  uint32_t lo = __shfl_xor(static_cast<uint32_t>(v), m, WAVE);
  uint32_t hi = __shfl_xor(static_cast<uint32_t>(v >> 32), m, WAVE);
  return (static_cast<uint64_t>(hi) << 32) | lo;
}

__device__ __forceinline__ uint64_t shfl_up_u64(uint64_t v, int d) {
  uint32_t lo = __shfl_up(static_cast<uint32_t>(v), d, WAVE);
  uint32_t hi = __shfl_up(static_cast<uint32_t>(v >> 32), d, WAVE);
  return (static_cast<uint64_t>(hi) << 32) | lo;
}

// Lane i receives lane i + 1's value; lane 63 keeps its own.  A data-parallel-primitive move over the whole wave
// (no LDS traffic); call it with all 64 lanes active.
__device__ __forceinline__ uint32_t from_next_lane(uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(static_cast<int>(v), static_cast<int>(v), 0x130, 0xf, 0xf, false));   // wave_shl:1
}

// Wave-wide reductions over all 64 lanes (result in every lane).
__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += shfl_xor_u64(v, m);
  return v;
}
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, WAVE);
  return v;
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) { uint32_t o = __shfl_xor(v, m, WAVE); v = o > v ? o : v; }
  return v;
}
__device__ __forceinline__ uint64_t wave_min_u64(uint64_t v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) { uint64_t o = shfl_xor_u64(v, m); v = o < v ? o : v; }
  return v;
}
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) { uint64_t o = shfl_xor_u64(v, m); v = o > v ? o : v; }
  return v;
}

// Inclusive prefix sum across the 64 lanes, with data-parallel-primitive moves (no LDS traffic):
// shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of row 0 / 2 is broadcast
// into the next row (rows 1 and 3), then the last lane of row 1 into rows 2 and 3.  Lanes without a
// source receive 0.  Must be called by all 64 lanes of the wave.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, ROW_MASK, 0xf, false));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint64_t dpp_or_zero_u64(uint64_t v) {
  const uint32_t lo = dpp_or_zero<CTRL, ROW_MASK>(static_cast<uint32_t>(v));
  const uint32_t hi = dpp_or_zero<CTRL, ROW_MASK>(static_cast<uint32_t>(v >> 32));
  return (static_cast<uint64_t>(hi) << 32) | lo;
}
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v) {
  v += dpp_or_zero<0x111, 0xf>(v);   // row_shr:1
  v += dpp_or_zero<0x112, 0xf>(v);   // row_shr:2
  v += dpp_or_zero<0x114, 0xf>(v);   // row_shr:4
  v += dpp_or_zero<0x118, 0xf>(v);   // row_shr:8
  v += dpp_or_zero<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
  v += dpp_or_zero<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
  return v;
}
__device__ __forceinline__ uint64_t wave_incl_scan_u64(uint64_t v) {
  v += dpp_or_zero_u64<0x111, 0xf>(v);
  v += dpp_or_zero_u64<0x112, 0xf>(v);
  v += dpp_or_zero_u64<0x114, 0xf>(v);
  v += dpp_or_zero_u64<0x118, 0xf>(v);
  v += dpp_or_zero_u64<0x142, 0xa>(v);
  v += dpp_or_zero_u64<0x143, 0xc>(v);
  return v;
}

// Exclusive prefix sum across a 256-thread block; returns this thread's exclusive prefix and
// the block total (in every thread).  `lds` needs 8 words.
__device__ __forceinline__ uint32_t block_excl_scan_256(uint32_t v, uint32_t* lds, uint32_t& total) {
  const uint32_t lane = lane_id(), w = threadIdx.x >> 6;
  const uint32_t incl = wave_incl_scan_u32(v);
  __syncthreads();  // protect lds reuse
  if (lane == 63) lds[w] = incl;
  __syncthreads();
  uint32_t base = 0;
  const uint32_t t0 = lds[0], t1 = lds[1], t2 = lds[2], t3 = lds[3];
  if (w > 0) base += t0;
  if (w > 1) base += t1;
  if (w > 2) base += t2;
  total = t0 + t1 + t2 + t3;
  return base + incl - v;
}

// Nearest rank: the ceil(K * count / 100)-th smallest, as a 0-based index (count >= 1).
__device__ __forceinline__ uint64_t rank_index(uint64_t k, uint64_t count) { return (k * count + 99) / 100 - 1; }
__device__ __forceinline__ uint32_t rank_index_u32(uint32_t k, uint32_t count) { return (k * count + 99) / 100 - 1; }

// Number of segment heads before sorted position pos (head bit mask + per-word prefix counts).
__device__ __forceinline__ uint32_t heads_before(const uint64_t* __restrict__ bits, const uint32_t* __restrict__ word_prefix,
                                                 uint64_t n, uint32_t n_heads, uint64_t pos) {
  if (pos >= n) return n_heads;
  const uint64_t w = pos >> 6;
  return word_prefix[w] + static_cast<uint32_t>(__popcll(bits[w] & ((1ull << (pos & 63)) - 1ull)));
}

// Appends one item per lane with `want` set to a list whose length lives at *counter; returns the
// lane's position (undefined for lanes without `want`).  One atomic per wave.  Call from all lanes.
__device__ __forceinline__ uint32_t wave_append(uint32_t* counter, bool want) {
  const uint64_t mask = ballot(want);
  if (mask == 0) return 0;
  const int leader = __builtin_ctzll(mask);
  uint32_t base = 0;
  if (lane_id() == static_cast<uint32_t>(leader)) base = atomicAdd(counter, static_cast<uint32_t>(__popcll(mask)));
  base = __shfl(base, leader, WAVE);
  return base + popc_below(mask);
}

// Workgroups are handed to the eight accelerator dies (XCDs) round robin by workgroup number.  Where
// one workgroup handles one task and neighbouring tasks differ a lot in cost (or alternate between
// "mine" and "not mine"), that would load the dies unevenly; this map gives every die a contiguous
// eighth of the items instead.  Launch xcd_grid(n) workgroups; items >= n do not exist.
constexpr uint32_t N_XCD = 8;
__host__ __device__ inline uint32_t xcd_grid(uint32_t n) { return ((n + N_XCD - 1) / N_XCD) * N_XCD; }
__device__ __forceinline__ uint32_t xcd_item(uint32_t block, uint32_t n) {
  const uint32_t per = (n + N_XCD - 1) / N_XCD;
  return (block % N_XCD) * per + block / N_XCD;
}

// Largest t in [0, n_tasks) with off[t] <= pos, skipping empty tasks to the one that owns pos
// (requires pos < off[n_tasks]).
__device__ __forceinline__ uint32_t task_of(const uint64_t* __restrict__ off, uint32_t n_tasks, uint64_t pos) {
  uint32_t lo = 0, hi = n_tasks;  // invariant: off[lo] <= pos < off[hi]
  while (hi - lo > 1) {
    uint32_t mid = lo + ((hi - lo) >> 1);
    if (off[mid] <= pos) lo = mid; else hi = mid;
  }
  return lo;
}

}  // namespace fikit
