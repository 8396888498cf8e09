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
// task, or my key differs from my left neighbour's".  A key below its left neighbour's inside a task
// means the task is not sorted (yet): ctrl->wide is raised.
__global__ void __launch_bounds__(256)
k_head_bits(const uint64_t* __restrict__ key, uint64_t n, const uint64_t* __restrict__ off, uint32_t n_tasks,
            const uint32_t* __restrict__ gflag, uint64_t* __restrict__ bits, Ctrl* ctrl) {
  const uint64_t i = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
  const uint64_t first = i - lane_id();  // the wave's first position (same in every lane)
  bool head = false;
  if (first < n) {
    uint32_t t = task_of(off, n_tasks, first);
    if (i < n) {
      while (off[t + 1] <= i) ++t;      // step over task boundaries inside the wave's window
      if (gflag[t]) {
        head = (i == off[t]) || (key[i] != key[i - 1]);
        if (i != off[t] && key[i] < key[i - 1]) atomicOr(&ctrl->wide, 1u);
      }
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
constexpr int BIG_THREADS = 256;      // rows of up to BIG_ROW_SPLIT samples
constexpr int HUGE_THREADS = 1024;    // longer rows
constexpr uint32_t BIG_ROW_SPLIT = 4096;

template <int THREADS>
struct BigSmem {
  uint32_t hist[2][256];
  uint64_t red[THREADS / WAVE][4];
  uint32_t aux[4];
  uint32_t sel_bin[2];
  uint64_t sel_k[2];
};

// Adds one to hist[bin] for every lane with `todo`.  Samples of one ID cluster: the lanes that share the
// bin of the wave's first pending lane add once, together (twice over); what is left adds one by one.
// Must be called by whole waves.
__device__ __forceinline__ void wave_hist_add(uint32_t* hist, bool todo, uint32_t bin, uint32_t lane) {
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    const uint64_t pending = ballot(todo);
    if (pending == 0) break;
    const int leader = __builtin_ctzll(pending);
    const uint32_t lead_bin = __shfl(bin, leader, WAVE);
    const uint64_t same = ballot(todo && bin == lead_bin);
    if (static_cast<int>(lane) == leader) atomicAdd(&hist[lead_bin], static_cast<uint32_t>(__popcll(same)));
    todo = todo && bin != lead_bin;
  }
  if (todo) atomicAdd(&hist[bin], 1u);
}

// The k50-th and the k95-th smallest (0-based) of vals[0..m) among samples != skip, by
// most-significant-digit radix selection, both in the same passes over the samples: histogram the
// current byte of the samples that agree with the bytes fixed so far (one histogram per rank once their
// fixed bytes differ), walk it to the bin that holds the rank, fix that byte, repeat.  The bytes above
// the highest byte in which the smallest and the largest sample differ are the same in all samples and
// are fixed from the start.
template <int THREADS>
__device__ __forceinline__ void block_select2(const int64_t* __restrict__ vals, uint32_t m, uint64_t k50, uint64_t k95,
                                              uint64_t minval, uint64_t maxval, bool skip_none, BigSmem<THREADS>& sm,
                                              uint64_t& p50, uint64_t& p95) {
  if (minval == maxval) { p50 = p95 = maxval; return; }
  const uint32_t tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const int top = (63 - __builtin_clzll(minval ^ maxval)) >> 3;
  const uint64_t common = top == 7 ? 0 : (maxval >> (8 * (top + 1))) << (8 * (top + 1));
  uint64_t prefix[2] = {common, common}, k[2] = {k50, k95};
  for (int byte = top; byte >= 0; --byte) {
    const int shift = 8 * byte;
    const bool split = prefix[0] != prefix[1];      // (the same in all threads)
    if (tid < 256) { sm.hist[0][tid] = 0; sm.hist[1][tid] = 0; }
    __syncthreads();
    // (whole waves stay in the loop: ballots inside; four loads are in flight per lane)
    for (uint32_t i0 = 0; i0 < m; i0 += 4 * THREADS) {
      int64_t sv4[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t i = i0 + u * THREADS + tid;
        sv4[u] = i < m ? vals[i] : GAP_NONE;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t i = i0 + u * THREADS + tid;
        const int64_t sv = sv4[u];
        const uint64_t v = static_cast<uint64_t>(sv);
        const bool in = i < m && !(skip_none && sv == GAP_NONE);
        const uint32_t bin = static_cast<uint32_t>(v >> shift) & 0xffu;
        const uint64_t above = byte == 7 ? 0 : v >> (shift + 8);
        wave_hist_add(sm.hist[0], in && (byte == 7 || above == prefix[0] >> (shift + 8)), bin, lane);
        if (split) wave_hist_add(sm.hist[1], in && (byte == 7 || above == prefix[1] >> (shift + 8)), bin, lane);
      }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      // exclusive prefix over the 256 bins (held by the first four waves), then the bin that holds rank k[q]
      const uint32_t c = tid < 256 ? sm.hist[split ? q : 0][tid] : 0u;
      const uint32_t incl = wave_incl_scan_u32(c);
      if (tid < 256 && lane == 63) sm.aux[w] = incl;
      __syncthreads();
      if (tid < 256) {
        uint32_t base = 0;
        for (uint32_t j = 0; j < w; ++j) base += sm.aux[j];
        const uint32_t ex = base + incl - c;
        if (k[q] >= ex && k[q] < static_cast<uint64_t>(ex) + c) { sm.sel_bin[q] = tid; sm.sel_k[q] = k[q] - ex; }
      }
      __syncthreads();
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      prefix[q] |= static_cast<uint64_t>(sm.sel_bin[q]) << shift;
      k[q] = sm.sel_k[q];
    }
    __syncthreads();
  }
  p50 = prefix[0];
  p95 = prefix[1];
}

template <int THREADS>
__device__ __forceinline__ StatsAcc block_stats(const int64_t* __restrict__ vals, uint32_t m, bool skip_none, BigSmem<THREADS>& sm) {
  const uint32_t tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  uint64_t cnt = 0, sum = 0, mn = ~0ull, mx = 0;
  for (uint32_t i0 = tid; i0 < m; i0 += 4 * THREADS) {      // (four loads in flight per lane)
    int64_t sv4[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) sv4[u] = i0 + u * THREADS < m ? vals[i0 + u * THREADS] : GAP_NONE;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t sv = sv4[u];
      const bool in = i0 + u * THREADS < m && !(skip_none && sv == GAP_NONE);
      const uint64_t v = static_cast<uint64_t>(sv);
      cnt += in ? 1u : 0u; sum += in ? v : 0u; mn = (in && v < mn) ? v : mn; mx = (in && v > mx) ? v : mx;
    }
  }
  cnt = wave_sum_u64(cnt); sum = wave_sum_u64(sum); mn = wave_min_u64(mn); mx = wave_max_u64(mx);
  __syncthreads();
  if (lane == 0) { sm.red[w][0] = cnt; sm.red[w][1] = sum; sm.red[w][2] = mn; sm.red[w][3] = mx; }
  __syncthreads();
  StatsAcc s;
  s.count = 0; s.sum = 0; s.mn = ~0ull; s.mx = 0;
  for (int j = 0; j < THREADS / WAVE; ++j) {
    s.count += sm.red[j][0];
    s.sum += sm.red[j][1];
    s.mn = min(s.mn, sm.red[j][2]);
    s.mx = max(s.mx, sm.red[j][3]);
  }
  if (s.count == 0) { s.sum = s.mn = s.mx = s.p50 = s.p95 = 0; return s; }
  block_select2<THREADS>(vals, m, rank_index(50, s.count), rank_index(95, s.count), s.mn, s.mx, skip_none, sm, s.p50, s.p95);
  return s;
}

// Work lists of the rows with long segments: rows of 65 .. BIG_ROW_SPLIT launches from the front of
// rlist (their number in ctrl->n_class[0]), longer ones from its back (ctrl->n_class[1]); both counters
// must be zero at the start.  Launching one workgroup per row and letting most of them return at once
// costs more than the rows themselves when rows are many.
__global__ void k_stats_lists(const uint32_t* __restrict__ seg_start, uint64_t n_rows, const uint64_t* __restrict__ off,
                              uint32_t n_tasks, uint32_t* __restrict__ rlist, Ctrl* ctrl) {
  const uint64_t r = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  uint32_t cls = 0;
  if (r < n_rows) {
    const uint32_t s = seg_start[r];
    const uint32_t task = task_of(off, n_tasks, s);
    const uint64_t task_end = off[task + 1];
    const uint32_t e = seg_start[r + 1] < task_end ? seg_start[r + 1] : static_cast<uint32_t>(task_end);
    const uint32_t m = e - s;
    cls = m <= 64 ? 0u : (m <= BIG_ROW_SPLIT ? 1u : 2u);
  }
  const uint32_t front = wave_append(&ctrl->n_class[0], cls == 1u);
  if (cls == 1u) rlist[front] = static_cast<uint32_t>(r);
  const uint32_t back = wave_append(&ctrl->n_class[1], cls == 2u);
  if (cls == 2u) rlist[n_rows - 1 - back] = static_cast<uint32_t>(r);
}

// Workgroups take the rows of one of the two lists in turn (from_back: the long rows).
template <int THREADS>
__global__ void __launch_bounds__(THREADS)
k_stats_big(const uint32_t* __restrict__ seg_start, uint64_t n_rows, const uint64_t* __restrict__ off, uint32_t n_tasks,
            const uint64_t* __restrict__ key, const int64_t* __restrict__ exec, const int64_t* __restrict__ gap,
            const uint64_t* __restrict__ bits, const uint32_t* __restrict__ word_prefix, uint64_t n,
            const uint32_t* __restrict__ row_off32, fikit_row* __restrict__ rows, const uint32_t* __restrict__ rlist,
            const uint32_t* __restrict__ count, uint32_t from_back) {
  __shared__ BigSmem<THREADS> sm;
  const uint32_t items = *count;
  for (uint32_t item = blockIdx.x; item < items; item += gridDim.x) {
    const uint64_t r = from_back ? rlist[n_rows - 1 - item] : rlist[item];
    const uint32_t s = seg_start[r];
    const uint32_t task = task_of(off, n_tasks, s);
    const uint64_t task_end = off[task + 1];
    const uint32_t e = seg_start[r + 1] < task_end ? seg_start[r + 1] : static_cast<uint32_t>(task_end);
    const uint32_t m = e - s;
    const StatsAcc es = block_stats<THREADS>(exec + s, m, false, sm);
    const StatsAcc gs = block_stats<THREADS>(gap + s, m, true, sm);
    if (threadIdx.x < 64) {
      const uint64_t id = key[s];
      const uint64_t dst = row_off32[task] + (r - heads_before(bits, word_prefix, n, static_cast<uint32_t>(n_rows), off[task]));
      write_row(rows + dst, id, task, es, gs);
    }
  }
}

}  // namespace fikit
