// Segment boundaries and per-(task, ID) statistics over the sorted launches: the set S_UID and,
// per unique ID, the reduction of its execution times K and idle times G (Section 3.2, the
// equations for SK_j and SG_j give sum / count; min, max and nearest-rank percentiles are
// reduced from the same samples).
#pragma once

#include "common.hip.h"

namespace fikit {

// ------------------------------------------------------------------ segment heads
// One bit per sorted position: set where a new (task, ID) group of a general-path task begins
// (positions of other tasks give 0).  A wave produces one 64-bit word with a ballot of "I start a
// task, or my key differs from my left neighbour's".
__global__ void __launch_bounds__(256)
k_head_bits(const uint64_t* __restrict__ key, uint64_t n, const uint64_t* __restrict__ off, uint32_t n_tasks,
            const uint32_t* __restrict__ gflag, uint64_t* __restrict__ bits) {
  const uint64_t i = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
  const uint64_t first = i - lane_id();  // the wave's first position (same in every lane)
  bool head = false;
  if (first < n) {
    uint32_t t = task_of(off, n_tasks, first);
    if (i < n) {
      while (off[t + 1] <= i) ++t;      // step over task boundaries inside the wave's window
      if (gflag[t]) head = (i == off[t]) || (key[i] != key[i - 1]);
    }
  }
  const uint64_t word = ballot(head);
  if (lane_id() == 0 && (i < n)) bits[i >> 6] = word;
}

__global__ void k_popcount_words(const uint64_t* __restrict__ bits, uint64_t n_words, uint32_t* __restrict__ out) {
  const uint64_t w = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (w < n_words) out[w] = static_cast<uint32_t>(__popcll(bits[w]));
}

// seg_start[r] = sorted position at which row r begins; seg_start[n_rows] = n.
__global__ void k_seg_starts(const uint64_t* __restrict__ bits, const uint32_t* __restrict__ word_prefix,
                             uint64_t n_words, uint64_t n, uint64_t n_rows, uint32_t* __restrict__ seg_start) {
  const uint64_t w = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (w == 0) seg_start[n_rows] = static_cast<uint32_t>(n);
  if (w >= n_words) return;
  uint64_t b = bits[w];
  uint32_t r = word_prefix[w];
  while (b) {
    const int bit = __builtin_ctzll(b);
    seg_start[r++] = static_cast<uint32_t>((w << 6) + bit);
    b &= b - 1;
  }
}

// Row count of every general-path task: heads inside its range of sorted positions.
__global__ void k_general_row_counts(const uint64_t* __restrict__ off, uint32_t n_tasks, const uint32_t* __restrict__ gflag,
                                     const uint64_t* __restrict__ bits, const uint32_t* __restrict__ word_prefix, uint64_t n,
                                     uint32_t n_heads, uint32_t* __restrict__ dcount) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (t >= n_tasks || !gflag[t]) return;
  dcount[t] = heads_before(bits, word_prefix, n, n_heads, off[t + 1]) - heads_before(bits, word_prefix, n, n_heads, off[t]);
}

__global__ void k_widen_offsets(const uint32_t* __restrict__ in, uint64_t count, uint64_t* __restrict__ out) {
  const uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < count) out[i] = in[i];
}

// ------------------------------------------------------------------ rows

struct StatsAcc {
  uint64_t count, sum, mn, mx, p50, p95;
};

// Writes one 128-byte row with the 16 first lanes of a wave (one 8-byte field each).
__device__ __forceinline__ void write_row(fikit_row* __restrict__ row, uint64_t id, uint32_t task, const StatsAcc& e,
                                          const StatsAcc& g) {
  const uint32_t l = lane_id();
  uint64_t v = 0;
  switch (l) {
    case 0: v = id; break;
    case 1: v = task; break;
    case 2: v = e.count; break;
    case 3: v = e.sum; break;
    case 4: v = e.mn; break;
    case 5: v = e.mx; break;
    case 6: v = e.p50; break;
    case 7: v = e.p95; break;
    case 8: v = g.count; break;
    case 9: v = g.sum; break;
    case 10: v = g.mn; break;
    case 11: v = g.mx; break;
    case 12: v = g.p50; break;
    case 13: v = g.p95; break;
    default: v = 0; break;
  }
  if (l < 16) reinterpret_cast<uint64_t*>(row)[l] = v;
}

// Statistics of up to 64 samples held one per lane (valid lanes only; samples are >= 0).
// Order statistics by counting: a sample's rank is the number of samples that precede it in
// (value, lane) order.
__device__ __forceinline__ StatsAcc wave_stats_le64(uint64_t v, bool valid, uint32_t m_lanes) {
  StatsAcc s;
  const uint64_t vmask = ballot(valid);
  s.count = static_cast<uint64_t>(__popcll(vmask));
  if (s.count == 0) { s.sum = s.mn = s.mx = s.p50 = s.p95 = 0; return s; }
  s.sum = wave_sum_u64(valid ? v : 0);
  s.mn = wave_min_u64(valid ? v : ~0ull);
  s.mx = wave_max_u64(valid ? v : 0);
  const uint32_t lane = lane_id();
  uint32_t rank = 0;
  for (uint32_t j = 0; j < m_lanes; ++j) {
    const uint64_t vj = shfl_u64(v, j);
    const bool vj_valid = (vmask >> j) & 1ull;
    if (vj_valid && (vj < v || (vj == v && j < lane))) ++rank;
  }
  const uint64_t k50 = rank_index(50, s.count), k95 = rank_index(95, s.count);
  const uint64_t b50 = ballot(valid && rank == k50), b95 = ballot(valid && rank == k95);
  s.p50 = shfl_u64(v, __builtin_ctzll(b50));
  s.p95 = shfl_u64(v, __builtin_ctzll(b95));
  return s;
}

// One wave per row whose segment has at most 64 launches.
__global__ void __launch_bounds__(256)
k_stats_small(const uint32_t* __restrict__ seg_start, uint64_t n_rows, const uint64_t* __restrict__ off, uint32_t n_tasks,
              const uint64_t* __restrict__ key, const int64_t* __restrict__ exec, const int64_t* __restrict__ gap,
              const uint64_t* __restrict__ bits, const uint32_t* __restrict__ word_prefix, uint64_t n,
              const uint32_t* __restrict__ row_off32, fikit_row* __restrict__ rows) {
  const uint64_t r = static_cast<uint64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (r >= n_rows) return;
  const uint32_t s = seg_start[r];
  const uint32_t task = task_of(off, n_tasks, s);
  // the next head may lie beyond tasks that do not take this path: a segment ends with its task
  const uint64_t task_end = off[task + 1];
  const uint32_t e = seg_start[r + 1] < task_end ? seg_start[r + 1] : static_cast<uint32_t>(task_end);
  const uint32_t m = e - s;
  if (m > 64) return;
  const uint32_t lane = lane_id();
  const bool in = lane < m;
  const uint64_t ev = in ? static_cast<uint64_t>(exec[s + lane]) : 0;
  const int64_t gv = in ? gap[s + lane] : GAP_NONE;
  const StatsAcc es = wave_stats_le64(ev, in, m);
  const StatsAcc gs = wave_stats_le64(static_cast<uint64_t>(gv), in && gv != GAP_NONE, m);
  const uint64_t id = key[s];
  // r counts general-path rows only; the row's final place is relative to its task's first row
  const uint64_t dst = row_off32[task] + (r - heads_before(bits, word_prefix, n, static_cast<uint32_t>(n_rows), off[task]));
  write_row(rows + dst, id, task, es, gs);
}

// ------------------------------------------------------------------ long segments
constexpr int BIG_THREADS = 256;

struct BigSmem {
  uint32_t hist[256];
  uint64_t red[4][8];
  uint32_t aux[8];
  uint32_t sel_bin;
  uint64_t sel_k;
};

// k-th smallest (0-based) of vals[0..m) among samples != skip, by most-significant-digit radix
// selection: histogram the current byte of the samples that agree with the bytes fixed so far,
// walk the histogram to the bin that holds rank k, fix that byte, repeat.
__device__ __forceinline__ uint64_t block_select(const int64_t* __restrict__ vals, uint32_t m, uint64_t k, uint64_t maxval,
                                                 bool skip_none, BigSmem& sm) {
  const uint32_t tid = threadIdx.x;
  int top = 7;
  while (top > 0 && ((maxval >> (8 * top)) & 0xff) == 0) --top;
  uint64_t prefix = 0;
  for (int byte = top; byte >= 0; --byte) {
    const int shift = 8 * byte;
    sm.hist[tid] = 0;
    __syncthreads();
    for (uint32_t i = tid; i < m; i += BIG_THREADS) {
      const int64_t sv = vals[i];
      if (skip_none && sv == GAP_NONE) continue;
      const uint64_t v = static_cast<uint64_t>(sv);
      const bool match = (byte == 7) ? true : ((v >> (shift + 8)) == (prefix >> (shift + 8)));
      if (match) atomicAdd(&sm.hist[(v >> shift) & 0xff], 1u);
    }
    __syncthreads();
    const uint32_t c = sm.hist[tid];
    uint32_t total;
    const uint32_t ex = block_excl_scan_256(c, sm.aux, total);
    if (k >= ex && k < static_cast<uint64_t>(ex) + c) { sm.sel_bin = tid; sm.sel_k = k - ex; }
    __syncthreads();
    prefix |= static_cast<uint64_t>(sm.sel_bin) << shift;
    k = sm.sel_k;
    __syncthreads();
  }
  return prefix;
}

__device__ __forceinline__ StatsAcc block_stats(const int64_t* __restrict__ vals, uint32_t m, bool skip_none, BigSmem& sm) {
  const uint32_t tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  uint64_t cnt = 0, sum = 0, mn = ~0ull, mx = 0;
  for (uint32_t i = tid; i < m; i += BIG_THREADS) {
    const int64_t sv = vals[i];
    if (skip_none && sv == GAP_NONE) continue;
    const uint64_t v = static_cast<uint64_t>(sv);
    ++cnt; sum += v; mn = v < mn ? v : mn; mx = v > mx ? v : mx;
  }
  cnt = wave_sum_u64(cnt); sum = wave_sum_u64(sum); mn = wave_min_u64(mn); mx = wave_max_u64(mx);
  __syncthreads();
  if (lane == 0) { sm.red[w][0] = cnt; sm.red[w][1] = sum; sm.red[w][2] = mn; sm.red[w][3] = mx; }
  __syncthreads();
  StatsAcc s;
  s.count = sm.red[0][0] + sm.red[1][0] + sm.red[2][0] + sm.red[3][0];
  s.sum = sm.red[0][1] + sm.red[1][1] + sm.red[2][1] + sm.red[3][1];
  s.mn = min(min(sm.red[0][2], sm.red[1][2]), min(sm.red[2][2], sm.red[3][2]));
  s.mx = max(max(sm.red[0][3], sm.red[1][3]), max(sm.red[2][3], sm.red[3][3]));
  if (s.count == 0) { s.sum = s.mn = s.mx = s.p50 = s.p95 = 0; return s; }
  s.p50 = block_select(vals, m, rank_index(50, s.count), s.mx, skip_none, sm);
  s.p95 = block_select(vals, m, rank_index(95, s.count), s.mx, skip_none, sm);
  return s;
}

// One workgroup per row whose segment has more than 64 launches.
__global__ void __launch_bounds__(BIG_THREADS)
k_stats_big(const uint32_t* __restrict__ seg_start, uint64_t n_rows, const uint64_t* __restrict__ off, uint32_t n_tasks,
            const uint64_t* __restrict__ key, const int64_t* __restrict__ exec, const int64_t* __restrict__ gap,
            const uint64_t* __restrict__ bits, const uint32_t* __restrict__ word_prefix, uint64_t n,
            const uint32_t* __restrict__ row_off32, fikit_row* __restrict__ rows) {
  __shared__ BigSmem sm;
  const uint64_t r = blockIdx.x;
  if (r >= n_rows) return;
  const uint32_t s = seg_start[r];
  const uint32_t task = task_of(off, n_tasks, s);
  const uint64_t task_end = off[task + 1];
  const uint32_t e = seg_start[r + 1] < task_end ? seg_start[r + 1] : static_cast<uint32_t>(task_end);
  const uint32_t m = e - s;
  if (m <= 64) return;
  const StatsAcc es = block_stats(exec + s, m, false, sm);
  const StatsAcc gs = block_stats(gap + s, m, true, sm);
  if (threadIdx.x < 64) {
    const uint64_t id = key[s];
    const uint64_t dst = row_off32[task] + (r - heads_before(bits, word_prefix, n, static_cast<uint32_t>(n_rows), off[task]));
    write_row(rows + dst, id, task, es, gs);
  }
}

}  // namespace fikit
