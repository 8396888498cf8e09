// Whole-task profiling in one workgroup, for tasks that are short and have few distinct Kernel
// IDs (the regime the paper describes: a service repeats the same kernels over and over).
//
// One workgroup reads a task's launch records once, and produces its rows without ever writing
// per-launch intermediates to memory:
//   1. Kernel ID (Section 3.2 "Identifying each kernel"), execution time K and idle time G of
//      every launch stay in registers; the IDs are also written out in launch order.
//   2. The task's set of unique IDs (S_UID, Section 3.2) is built in an LDS hash table, then
//      ranked so that rows come out in ascending ID order.
//   3. count / sum / min / max per ID (sum / count = SK_j, SG_j of Section 3.2) by LDS atomics.
//   4. Nearest-rank p50 / p95 per ID by most-significant-digit radix selection: per pass, every
//      launch whose value still agrees with the digits fixed so far for its ID adds one to that
//      ID's digit histogram in LDS; one thread per (ID, percentile) then walks the histogram to
//      the digit that holds the wanted rank.  All IDs of the task advance together.
//
// Rows are staged in the task's own slice of two workspace arrays and moved to their final
// place once every task's row count is known.  A task that does not fit (too many distinct IDs)
// writes its per-launch values to the workspace arrays instead and is flagged for the general
// sort-based path.
#pragma once

#include "common.hip.h"
#include "profile_kernels.hip.h"

namespace fikit {

constexpr uint64_t HT_EMPTY = ~0ull;
constexpr uint32_t FUSE_SMALL_MAX = 4096;    // tasks up to this many launches: 256-thread workgroup
constexpr uint32_t FUSE_MAX = 16384;         // tasks up to this many launches: 1024-thread workgroup

template <int NT>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* aux, uint32_t& total) {
  constexpr int NW = NT / WAVE;
  const uint32_t lane = lane_id(), w = threadIdx.x >> 6;
  const uint32_t incl = wave_incl_scan_u32(v);
  __syncthreads();
  if (lane == 63) aux[w] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int k = 0; k < NW; ++k) {
    const uint32_t s = aux[k];
    if (static_cast<uint32_t>(k) < w) base += s;
    tot += s;
  }
  total = tot;
  return base + incl - v;
}

template <int NT, int DMAX, int HIST_WORDS>
struct FusedSmem {
  static constexpr int HT = 2 * DMAX;
  uint64_t ht_key[HT];
  uint32_t ht_cnt[HT];
  uint16_t slot_rank[HT];
  uint64_t rkey[DMAX];
  uint32_t rcnt[DMAX];
  uint32_t gcnt[DMAX];
  uint64_t pref[4][DMAX];
  uint16_t kth[4][DMAX];
  union {
    struct { uint64_t ckey[DMAX]; uint32_t cslot[DMAX]; } tmp;
    struct { uint64_t esum[DMAX], emin[DMAX], emax[DMAX], gsum[DMAX], gmin[DMAX], gmax[DMAX]; } acc;
    uint32_t hist[HIST_WORDS];
  } u;
  uint64_t maxv;
  uint32_t aux[NT / WAVE];
  uint32_t ndist;
  uint32_t fallback;
};

// Where row j of a task is staged: the task's slice of stage_a, then its slice of stage_b.
__device__ __forceinline__ uint64_t* staged_row(int64_t* stage_a, int64_t* stage_b, uint64_t base, uint32_t m, uint32_t j) {
  const uint32_t cap1 = m >> 4;  // rows of 16 words that fit in m words
  return j < cap1 ? reinterpret_cast<uint64_t*>(stage_a + base) + static_cast<uint64_t>(j) * 16
                  : reinterpret_cast<uint64_t*>(stage_b + base) + static_cast<uint64_t>(j - cap1) * 16;
}

template <int NT, int KPT, int DMAX, int HIST_WORDS>
__global__ void __launch_bounds__(NT)
k_task_fused(const fikit_launch* __restrict__ rec, const uint64_t* __restrict__ off, uint32_t min_len, uint32_t max_len,
             uint64_t* __restrict__ ids, int64_t* __restrict__ e0, int64_t* __restrict__ g0,
             int64_t* __restrict__ stage_a, int64_t* __restrict__ stage_b, uint32_t* __restrict__ dcount,
             uint32_t* __restrict__ gflag, Ctrl* ctrl) {
  using Smem = FusedSmem<NT, DMAX, HIST_WORDS>;
  constexpr int HT = Smem::HT;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);
  if (ctrl->status & ERR_OFFSETS) return;
  const uint32_t t = blockIdx.x;
  const uint64_t base = off[t];
  const uint64_t len64 = off[t + 1] - base;
  if (len64 < min_len || len64 > max_len) return;
  const uint32_t m = static_cast<uint32_t>(len64);
  const uint32_t tid = threadIdx.x;

  for (uint32_t i = tid; i < HT; i += NT) { sm.ht_key[i] = HT_EMPTY; sm.ht_cnt[i] = 0; }
  if (tid == 0) { sm.ndist = 0; sm.fallback = 0; sm.maxv = 0; }
  __syncthreads();

  // ---- 1. read, hash, measure; 2a. insert IDs ---------------------------------------------
  uint64_t ev[KPT], gv[KPT];   // execution time, idle time (GAP_NONE for the task's last launch)
  uint32_t sl[KPT];            // hash slot, later the rank of the launch's ID
  uint64_t my_max = 0;
  bool bad = false;
#pragma unroll
  for (int r = 0; r < KPT; ++r) {
    ev[r] = 0; gv[r] = static_cast<uint64_t>(GAP_NONE); sl[r] = 0;
    if (static_cast<uint32_t>(r) * NT < m) {
      const uint32_t i = r * NT + tid;
      if (i < m) {
        const uint4* p = reinterpret_cast<const uint4*>(rec + base + i);
        const uint4 a = p[0], b = p[1], c = p[2];
        int64_t next_start = 0;
        const bool has_next = (i + 1 < m);
        if (has_next) next_start = rec[base + i + 1].start_ns;
        const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        const uint64_t id = kernel_id_of(w);
        const int64_t start = static_cast<int64_t>((static_cast<uint64_t>(c.y) << 32) | c.x);
        const int64_t end = static_cast<int64_t>((static_cast<uint64_t>(c.w) << 32) | c.z);
        bad |= (end < start);
        ev[r] = static_cast<uint64_t>(end - start);
        if (has_next) { const int64_t g = next_start - end; gv[r] = static_cast<uint64_t>(g < 0 ? 0 : g); }
        ids[base + i] = id;
        my_max = ev[r] > my_max ? ev[r] : my_max;
        if (has_next) my_max = gv[r] > my_max ? gv[r] : my_max;
        // open addressing, linear probing; the ID is already a hash
        uint32_t h = (static_cast<uint32_t>(id >> 32) ^ static_cast<uint32_t>(id)) & (HT - 1);
        bool placed = false;
        if (id != HT_EMPTY) {
          for (int probe = 0; probe < HT; ++probe) {
            const uint64_t k = __hip_atomic_load(&sm.ht_key[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (k == id) { placed = true; break; }
            if (k == HT_EMPTY) {
              const uint64_t old = atomicCAS(reinterpret_cast<unsigned long long*>(&sm.ht_key[h]), HT_EMPTY, id);
              if (old == HT_EMPTY) { atomicAdd(&sm.ndist, 1u); placed = true; break; }
              if (old == id) { placed = true; break; }
            }
            h = (h + 1) & (HT - 1);
          }
        }
        if (placed) atomicAdd(&sm.ht_cnt[h], 1u); else atomicOr(&sm.fallback, 1u);
        sl[r] = h;
      }
    }
  }
  if (bad) atomicOr(&ctrl->status, ERR_BAD_RECORD);
  my_max = wave_max_u64(my_max);
  if (lane_id() == 0) atomicMax(reinterpret_cast<unsigned long long*>(&sm.maxv), my_max);
  __syncthreads();
  const uint32_t D = sm.ndist;
  if (sm.fallback || D > DMAX || D > 2 * (m >> 4)) {
    // general path: hand over the per-launch values
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
      const uint32_t i = r * NT + tid;
      if (i < m) { e0[base + i] = static_cast<int64_t>(ev[r]); g0[base + i] = static_cast<int64_t>(gv[r]); }
    }
    if (tid == 0) { gflag[t] = 1; atomicAdd(reinterpret_cast<unsigned long long*>(&ctrl->n_general), 1ull); }
    return;
  }

  // ---- 2b. rank the distinct IDs -----------------------------------------------------------
  {
    uint32_t mine = 0;
    for (uint32_t s = tid; s < HT; s += NT) mine += (sm.ht_key[s] != HT_EMPTY);
    uint32_t total;
    uint32_t at = block_excl_scan<NT>(mine, sm.aux, total);
    for (uint32_t s = tid; s < HT; s += NT)
      if (sm.ht_key[s] != HT_EMPTY) { sm.u.tmp.ckey[at] = sm.ht_key[s]; sm.u.tmp.cslot[at] = s; ++at; }
    __syncthreads();
    for (uint32_t j = tid; j < D; j += NT) {
      const uint64_t k = sm.u.tmp.ckey[j];
      uint32_t rank = 0;
      for (uint32_t i = 0; i < D; ++i) rank += (sm.u.tmp.ckey[i] < k);
      const uint32_t s = sm.u.tmp.cslot[j];
      sm.slot_rank[s] = static_cast<uint16_t>(rank);
      sm.rkey[rank] = k;
      sm.rcnt[rank] = sm.ht_cnt[s];
    }
    __syncthreads();
  }
#pragma unroll
  for (int r = 0; r < KPT; ++r) sl[r] = sm.slot_rank[sl[r]];
  __syncthreads();  // tmp (ckey/cslot) is dead from here on; acc reuses the space

  // ---- 3. count / sum / min / max per ID ----------------------------------------------------
  for (uint32_t j = tid; j < D; j += NT) {
    sm.u.acc.esum[j] = 0; sm.u.acc.emin[j] = ~0ull; sm.u.acc.emax[j] = 0;
    sm.u.acc.gsum[j] = 0; sm.u.acc.gmin[j] = ~0ull; sm.u.acc.gmax[j] = 0;
    sm.gcnt[j] = 0;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < KPT; ++r) {
    const uint32_t i = r * NT + tid;
    if (i < m) {
      const uint32_t j = sl[r];
      atomicAdd(reinterpret_cast<unsigned long long*>(&sm.u.acc.esum[j]), ev[r]);
      atomicMin(reinterpret_cast<unsigned long long*>(&sm.u.acc.emin[j]), ev[r]);
      atomicMax(reinterpret_cast<unsigned long long*>(&sm.u.acc.emax[j]), ev[r]);
      if (gv[r] != static_cast<uint64_t>(GAP_NONE)) {
        atomicAdd(&sm.gcnt[j], 1u);
        atomicAdd(reinterpret_cast<unsigned long long*>(&sm.u.acc.gsum[j]), gv[r]);
        atomicMin(reinterpret_cast<unsigned long long*>(&sm.u.acc.gmin[j]), gv[r]);
        atomicMax(reinterpret_cast<unsigned long long*>(&sm.u.acc.gmax[j]), gv[r]);
      }
    }
  }
  __syncthreads();
  for (uint32_t j = tid; j < D; j += NT) {
    uint64_t* row = staged_row(stage_a, stage_b, base, m, j);
    const uint32_t ec = sm.rcnt[j], gc = sm.gcnt[j];
    row[0] = sm.rkey[j];
    row[1] = t;
    row[2] = ec; row[3] = sm.u.acc.esum[j]; row[4] = sm.u.acc.emin[j]; row[5] = sm.u.acc.emax[j];
    row[8] = gc; row[9] = sm.u.acc.gsum[j];
    row[10] = gc ? sm.u.acc.gmin[j] : 0; row[11] = gc ? sm.u.acc.gmax[j] : 0;
    row[14] = 0; row[15] = 0;
    sm.kth[0][j] = static_cast<uint16_t>(rank_index_u32(50, ec));
    sm.kth[1][j] = static_cast<uint16_t>(rank_index_u32(95, ec));
    sm.kth[2][j] = static_cast<uint16_t>(gc ? rank_index_u32(50, gc) : 0);
    sm.kth[3][j] = static_cast<uint16_t>(gc ? rank_index_u32(95, gc) : 0);
    sm.pref[0][j] = 0; sm.pref[1][j] = 0; sm.pref[2][j] = 0; sm.pref[3][j] = 0;
  }
  __syncthreads();  // acc is dead from here on; hist reuses the space

  // ---- 4. nearest-rank percentiles by radix selection ---------------------------------------
  for (uint32_t i = tid; i < HIST_WORDS; i += NT) sm.u.hist[i] = 0;
  const uint64_t maxv = sm.maxv;
  const int nbits = maxv ? 64 - __builtin_clzll(maxv) : 1;
  // 16-bit counters, two per word: bins available per (ID, percentile) pair
  int B = 31 - __builtin_clz(static_cast<uint32_t>(HIST_WORDS * 2) / (4 * D));
  B = B > 8 ? 8 : B;
  const uint32_t bins = 1u << B;
  const int passes = (nbits + B - 1) / B;
  __syncthreads();
  for (int p = passes - 1; p >= 0; --p) {
    const int shift = p * B;
    const int hi = shift + B;
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
      const uint32_t i = r * NT + tid;
      if (i < m) {
        const uint32_t j = sl[r];
#pragma unroll
        for (int tg = 0; tg < 4; ++tg) {
          const uint64_t v = tg < 2 ? ev[r] : gv[r];
          if (tg >= 2 && v == static_cast<uint64_t>(GAP_NONE)) continue;
          const uint64_t pf = sm.pref[tg][j];
          const bool match = hi >= 64 ? true : (((v ^ pf) >> hi) == 0);
          if (match) {
            const uint32_t idx = ((tg * D + j) << B) + (static_cast<uint32_t>(v >> shift) & (bins - 1));
            atomicAdd(&sm.u.hist[idx >> 1], (idx & 1u) ? 0x10000u : 1u);
          }
        }
      }
    }
    __syncthreads();
    for (uint32_t q = tid; q < 4 * D; q += NT) {
      const uint32_t tg = q / D, j = q - tg * D;
      uint32_t k = sm.kth[tg][j];
      uint32_t cum = 0, digit = 0, knew = 0;
      bool found = false;
      const uint32_t w0 = (q << B) >> 1;
      for (uint32_t wd = 0; wd < (bins >> 1); ++wd) {
        const uint32_t pair = sm.u.hist[w0 + wd];
        sm.u.hist[w0 + wd] = 0;
        const uint32_t c0 = pair & 0xffffu, c1 = pair >> 16;
        if (!found && k < cum + c0) { found = true; digit = 2 * wd; knew = k - cum; }
        cum += c0;
        if (!found && k < cum + c1) { found = true; digit = 2 * wd + 1; knew = k - cum; }
        cum += c1;
      }
      if (found) {
        sm.kth[tg][j] = static_cast<uint16_t>(knew);
        sm.pref[tg][j] |= static_cast<uint64_t>(digit) << shift;
      }
    }
    __syncthreads();
  }
  for (uint32_t j = tid; j < D; j += NT) {
    uint64_t* row = staged_row(stage_a, stage_b, base, m, j);
    row[6] = sm.pref[0][j]; row[7] = sm.pref[1][j];
    row[12] = sm.pref[2][j]; row[13] = sm.pref[3][j];
  }
  if (tid == 0) dcount[t] = D;
}

// Moves a task's staged rows to their final place once the row offsets are known.
__global__ void __launch_bounds__(256)
k_gather_rows(const uint64_t* __restrict__ off, const uint32_t* __restrict__ row_off32, const uint32_t* __restrict__ gflag,
              const int64_t* __restrict__ stage_a, const int64_t* __restrict__ stage_b, fikit_row* __restrict__ rows) {
  const uint32_t t = blockIdx.x;
  if (gflag[t]) return;
  const uint32_t r0 = row_off32[t], D = row_off32[t + 1] - r0;
  if (D == 0) return;
  const uint64_t base = off[t];
  const uint32_t m = static_cast<uint32_t>(off[t + 1] - base);
  uint64_t* out = reinterpret_cast<uint64_t*>(rows + r0);
  for (uint32_t x = threadIdx.x; x < D * 16; x += 256) {
    const uint32_t j = x >> 4, f = x & 15;
    out[x] = staged_row(const_cast<int64_t*>(stage_a), const_cast<int64_t*>(stage_b), base, m, j)[f];
  }
}

}  // namespace fikit
