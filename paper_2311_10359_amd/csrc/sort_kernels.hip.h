// Grouping launches by (task, Kernel ID): least-significant-digit radix sort of every task's
// records on the 64-bit ID, carrying execution time and idle time as payload.  This realises
// the "uniquify" step that forms S_UID (Section 3.2): after it, equal IDs of a task are adjacent
// and IDs ascend.
//
//   - tasks of at most LEAF records are sorted entirely in LDS by one workgroup (k_leaf_sort);
//   - longer tasks are sorted one 8-bit digit per pass, a pass being ONE launch over tiles:
//       k_digit_hist     one read of the keys gives every task's digit counts for four passes at once
//       k_digit_bases    their exclusive prefix sums = where every digit's bucket starts in the task
//       k_onesweep_pass  per tile: rank the keys inside the tile (LDS), learn how many keys with each
//                        digit the task's earlier tiles hold by looking back at what those tiles have
//                        published (a chained scan: no histogram pass, no scan launches), and move
//                        (key, execution time, idle time) to its place through LDS so that writes leave
//                        in runs.
//
// Ranking inside a tile uses wavefront ballots: the lanes that hold the same digit find each
// other with eight ballots, so ranks are stable without sorting.
#pragma once

#include "common.hip.h"

namespace fikit {

// ------------------------------------------------------------------ device-wide exclusive scan
constexpr int SCAN_BLOCK = 256;
constexpr int SCAN_ITEMS = 16;
constexpr int SCAN_TILE = SCAN_BLOCK * SCAN_ITEMS;

__global__ void __launch_bounds__(SCAN_BLOCK)
k_scan_reduce(const uint32_t* __restrict__ in, uint64_t count, uint32_t* __restrict__ block_sums) {
  __shared__ uint32_t lds[8];
  const uint64_t base = static_cast<uint64_t>(blockIdx.x) * SCAN_TILE + static_cast<uint64_t>(threadIdx.x) * SCAN_ITEMS;
  uint32_t s = 0;
#pragma unroll
  for (int k = 0; k < SCAN_ITEMS; ++k) if (base + k < count) s += in[base + k];
  s = wave_sum_u32(s);
  if (lane_id() == 0) lds[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) block_sums[blockIdx.x] = lds[0] + lds[1] + lds[2] + lds[3];
}

// One workgroup turns the per-block sums into exclusive prefixes; writes the grand total.
__global__ void __launch_bounds__(SCAN_BLOCK)
k_scan_spine(uint32_t* __restrict__ block_sums, uint64_t nb, uint64_t* __restrict__ total_out) {
  __shared__ uint32_t lds[8];
  uint64_t carry = 0;
  for (uint64_t b0 = 0; b0 < nb; b0 += SCAN_BLOCK) {
    const uint64_t i = b0 + threadIdx.x;
    const uint32_t v = i < nb ? block_sums[i] : 0;
    uint32_t total;
    const uint32_t ex = block_excl_scan_256(v, lds, total);
    if (i < nb) block_sums[i] = static_cast<uint32_t>(carry) + ex;
    carry += total;
  }
  if (threadIdx.x == 0 && total_out) *total_out = carry;
}

__global__ void __launch_bounds__(SCAN_BLOCK)
k_scan_apply(uint32_t* __restrict__ data, uint64_t count, const uint32_t* __restrict__ block_sums) {
  __shared__ uint32_t lds[8];
  const uint64_t base = static_cast<uint64_t>(blockIdx.x) * SCAN_TILE + static_cast<uint64_t>(threadIdx.x) * SCAN_ITEMS;
  uint32_t v[SCAN_ITEMS];
  uint32_t s = 0;
#pragma unroll
  for (int k = 0; k < SCAN_ITEMS; ++k) { v[k] = (base + k < count) ? data[base + k] : 0; s += v[k]; }
  uint32_t total;
  uint32_t run = block_sums[blockIdx.x] + block_excl_scan_256(s, lds, total);
#pragma unroll
  for (int k = 0; k < SCAN_ITEMS; ++k) { if (base + k < count) data[base + k] = run; run += v[k]; }
}

// ------------------------------------------------------------------ sort plan
constexpr uint32_t LEAF = 8192;        // largest task sorted in LDS by one workgroup
constexpr int LEAF_THREADS = 1024;
constexpr int LEAF_WAVES = LEAF_THREADS / WAVE;
constexpr int LEAF_KPT = LEAF / LEAF_THREADS;

constexpr uint32_t TILE = 8192;  // records per tile of the multi-pass path
constexpr int TILE_THREADS = 512;
constexpr int TILE_WAVES = TILE_THREADS / WAVE;
constexpr int TILE_KPT = TILE / TILE_THREADS;

// tiles[t] = number of tiles task t contributes to the multi-pass path (0 for LDS-sorted tasks and
// for tasks that do not take the general path at all).
// tiles has n_tasks + 1 entries; the last is 0 so that an exclusive scan leaves the total there.
__global__ void k_plan_tiles(const uint64_t* __restrict__ off, uint32_t n_tasks, const uint32_t* __restrict__ gflag,
                             uint32_t* __restrict__ tiles, const Ctrl* ctrl) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (t > n_tasks) return;
  uint32_t v = 0;
  if (t < n_tasks && !(ctrl->status & ERR_OFFSETS)) {
    const uint64_t len = off[t + 1] - off[t];
    if (gflag[t] && len > LEAF) v = static_cast<uint32_t>((len + TILE - 1) / TILE);
  }
  tiles[t] = v;
}

// Task that owns multi-pass tile j: the t with tile_prefix[t] <= j < tile_prefix[t+1].
__device__ __forceinline__ uint32_t task_of_tile(const uint32_t* __restrict__ tile_prefix, uint32_t n_tasks, uint32_t j) {
  uint32_t lo = 0, hi = n_tasks;  // tile_prefix[lo] <= j < tile_prefix[hi]
  while (hi - lo > 1) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    if (tile_prefix[mid] <= j) lo = mid; else hi = mid;
  }
  return lo;
}

// ------------------------------------------------------------------ ranking by an 8-bit digit
// Rank of this lane's key among the keys with the same digit that the wave has seen so far
// (earlier rounds, then lower lanes).  cnt_w[256] is the wave's running digit count in LDS.
__device__ __forceinline__ uint32_t wave_rank_digit(uint32_t digit, bool valid, uint32_t* cnt_w) {
  uint64_t same = ballot(valid);
#pragma unroll
  for (int b = 0; b < 8; ++b) {
    const bool bit = (digit >> b) & 1u;
    const uint64_t bal = ballot(bit);
    same &= bit ? bal : ~bal;
  }
  uint32_t rank = 0;
  if (valid) {
    const uint32_t before = cnt_w[digit];
    rank = before + popc_below(same);
    if ((same >> lane_id()) == 1ull) cnt_w[digit] = before + static_cast<uint32_t>(__popcll(same));
  }
  __builtin_amdgcn_wave_barrier();
  return rank;
}

// After all waves have counted: turns cnt[w][d] into the tile-local start of (digit d, wave w)
// in (digit, wave) order.  Called by every thread of the block; NW waves.  `aux` needs 8 words.
// If digit_total is not null, thread d < 256 also stores the tile's count of digit d there.
template <int NW>
__device__ __forceinline__ void tile_digit_offsets(uint32_t (*cnt)[256], uint32_t* aux, uint32_t* digit_total) {
  __syncthreads();
  uint32_t tot = 0;
  const uint32_t d = threadIdx.x;
  if (d < 256) {
#pragma unroll 4
    for (int w = 0; w < NW; ++w) { const uint32_t c = cnt[w][d]; cnt[w][d] = tot; tot += c; }
    if (digit_total) digit_total[d] = tot;
  }
  // exclusive scan of the 256 digit totals (threads >= 256 contribute 0)
  const uint32_t lane = lane_id(), w = threadIdx.x >> 6;
  const uint32_t incl = wave_incl_scan_u32(tot);
  if (lane == 63 && w < 4) aux[w] = incl;
  __syncthreads();
  if (d < 256) {
    uint32_t base = incl - tot;
    if (w > 0) base += aux[0];
    if (w > 1) base += aux[1];
    if (w > 2) base += aux[2];
#pragma unroll 4
    for (int ww = 0; ww < NW; ++ww) cnt[ww][d] += base;
  }
  __syncthreads();
}

// ------------------------------------------------------------------ LDS sort of a short task
// One workgroup per task of 1..LEAF records.  Sorts (key, local index) by eight 8-bit passes in
// LDS, then writes the sorted keys and gathers the payload in the sorted order (in place, keys too if
// key_in == key_out: every key is in LDS and every payload value in a register before the first one is overwritten).
struct LeafSmem {
  uint64_t key[LEAF];
  uint32_t cnt[LEAF_WAVES][256];
  uint16_t idx[LEAF];
  uint32_t aux[8];
};

__global__ void __launch_bounds__(LEAF_THREADS)
k_leaf_sort(const uint64_t* __restrict__ off, uint32_t n_tasks, const uint32_t* __restrict__ gflag, const uint64_t* key_in,
            uint64_t* key_out, int64_t* __restrict__ exec_io, int64_t* __restrict__ gap_io,
            const Ctrl* ctrl) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  LeafSmem& sm = *reinterpret_cast<LeafSmem*>(smem_raw);
  if (ctrl->status & ERR_OFFSETS) return;
  const uint32_t t = xcd_item(blockIdx.x, n_tasks);
  if (t >= n_tasks || !gflag[t]) return;
  const uint64_t base = off[t];
  const uint64_t len64 = off[t + 1] - base;
  if (len64 == 0 || len64 > LEAF) return;
  const uint32_t m = static_cast<uint32_t>(len64);
  const uint32_t tid = threadIdx.x, lane = lane_id(), w = tid >> 6;

  for (uint32_t i = tid; i < m; i += LEAF_THREADS) { sm.key[i] = key_in[base + i]; sm.idx[i] = static_cast<uint16_t>(i); }
  // every wave owns `rounds` consecutive groups of 64 positions
  const uint32_t rounds = (m + LEAF_THREADS - 1) / LEAF_THREADS;
  const uint32_t wave_base = w * rounds * WAVE;
  __syncthreads();

  for (int pass = 0; pass < 8; ++pass) {
    const int shift = 8 * pass;
    for (uint32_t d = lane; d < 256; d += WAVE) sm.cnt[w][d] = 0;
    __builtin_amdgcn_wave_barrier();
    uint64_t k[LEAF_KPT];
    uint16_t ix[LEAF_KPT];
    uint32_t rk[LEAF_KPT];
#pragma unroll
    for (int r = 0; r < LEAF_KPT; ++r) {
      if (static_cast<uint32_t>(r) < rounds) {  // uniform across the block
        const uint32_t pos = wave_base + r * WAVE + lane;
        const bool valid = pos < m;
        k[r] = valid ? sm.key[pos] : 0;
        ix[r] = valid ? sm.idx[pos] : 0;
        rk[r] = wave_rank_digit(static_cast<uint32_t>(k[r] >> shift) & 0xffu, valid, sm.cnt[w]);
      }
    }
    tile_digit_offsets<LEAF_WAVES>(sm.cnt, sm.aux, nullptr);
#pragma unroll
    for (int r = 0; r < LEAF_KPT; ++r) {
      if (static_cast<uint32_t>(r) < rounds) {
        const uint32_t pos = wave_base + r * WAVE + lane;
        if (pos < m) {
          const uint32_t dst = sm.cnt[w][static_cast<uint32_t>(k[r] >> shift) & 0xffu] + rk[r];
          sm.key[dst] = k[r];
          sm.idx[dst] = ix[r];
        }
      }
    }
    __syncthreads();
  }

  int64_t e[LEAF_KPT], g[LEAF_KPT];
#pragma unroll
  for (int r = 0; r < LEAF_KPT; ++r) {
    const uint32_t i = tid + r * LEAF_THREADS;
    if (i < m) {
      const uint32_t src = sm.idx[i];
      e[r] = exec_io[base + src];
      g[r] = gap_io[base + src];
      key_out[base + i] = sm.key[i];
    } else {
      e[r] = 0;
      g[r] = 0;
    }
  }
  // all gathered values must have arrived in registers before anyone overwrites the source
#pragma unroll
  for (int r = 0; r < LEAF_KPT; ++r) asm volatile("" ::"v"(e[r]), "v"(g[r]));
  __syncthreads();
#pragma unroll
  for (int r = 0; r < LEAF_KPT; ++r) {
    const uint32_t i = tid + r * LEAF_THREADS;
    if (i < m) { exec_io[base + i] = e[r]; gap_io[base + i] = g[r]; }
  }
}

// ------------------------------------------------------------------ multi-pass path
constexpr int SORT_PASSES_PER_ROUND = 4;       // digit counts are taken for this many passes at once
constexpr uint32_t DIGIT_WORDS_PER_TILE = SORT_PASSES_PER_ROUND * 256 / 2;   // a task on this path has at least two tiles

// Digit counts of four passes (key bytes first_byte .. first_byte + 3) of every task on the multi-pass path:
// counts[(first tile of the task) * DIGIT_WORDS_PER_TILE + pass * 256 + digit].  The array must be zero.
__global__ void __launch_bounds__(256)
k_digit_hist(const uint64_t* __restrict__ off, uint32_t n_tasks, const uint32_t* __restrict__ tile_prefix,
             const uint64_t* __restrict__ keys, int first_byte, uint32_t* __restrict__ counts) {
  // (a few copies of every counter, one per group of lanes: a frequent key would otherwise serialise a wave on one address)
  constexpr int COPIES = 8;
  __shared__ uint32_t hist[SORT_PASSES_PER_ROUND][COPIES][256];
  const uint32_t j = blockIdx.x;
  const uint32_t t = task_of_tile(tile_prefix, n_tasks, j);
  const uint32_t tp = tile_prefix[t];
  const uint64_t start = off[t] + static_cast<uint64_t>(j - tp) * TILE;
  const uint64_t end = off[t + 1];
  const uint32_t m = static_cast<uint32_t>(end - start < TILE ? end - start : TILE);
  for (uint32_t x = threadIdx.x; x < SORT_PASSES_PER_ROUND * COPIES * 256; x += 256) (&hist[0][0][0])[x] = 0;
  __syncthreads();
  const uint32_t copy = threadIdx.x % COPIES;
  for (uint32_t i = threadIdx.x; i < m; i += 256) {
    const uint32_t k = static_cast<uint32_t>(keys[start + i] >> (8 * first_byte));
#pragma unroll
    for (int p = 0; p < SORT_PASSES_PER_ROUND; ++p) atomicAdd(&hist[p][copy][(k >> (8 * p)) & 0xffu], 1u);
  }
  __syncthreads();
  uint32_t* out = counts + static_cast<uint64_t>(tp) * DIGIT_WORDS_PER_TILE;
#pragma unroll
  for (int p = 0; p < SORT_PASSES_PER_ROUND; ++p) {
    uint32_t c = 0;
#pragma unroll
    for (int q = 0; q < COPIES; ++q) c += hist[p][q][threadIdx.x];
    if (c) atomicAdd(&out[p * 256 + threadIdx.x], c);
  }
}

// Turns every task's digit counts into exclusive prefix sums, pass by pass (one workgroup per task).
__global__ void __launch_bounds__(256)
k_digit_bases(uint32_t n_tasks, const uint32_t* __restrict__ tile_prefix, uint32_t* __restrict__ counts) {
  __shared__ uint32_t aux[8];
  const uint32_t t = blockIdx.x;
  if (t >= n_tasks || tile_prefix[t + 1] == tile_prefix[t]) return;
  uint32_t* c = counts + static_cast<uint64_t>(tile_prefix[t]) * DIGIT_WORDS_PER_TILE;
  for (int p = 0; p < SORT_PASSES_PER_ROUND; ++p) {
    uint32_t total;
    const uint32_t before = block_excl_scan_256(c[p * 256 + threadIdx.x], aux, total);
    c[p * 256 + threadIdx.x] = before;
  }
}

// What a tile publishes per digit for the tiles after it: first how many keys with the digit it holds itself, later how
// many the task holds up to and including it.  The state sits in the top two bits, the count below.
constexpr unsigned long long LOOK_EMPTY = 0ull, LOOK_OWN = 1ull << 62, LOOK_UPTO = 2ull << 62, LOOK_COUNT = (1ull << 62) - 1;
constexpr uint32_t LOOK_SPIN_LIMIT = 1u << 24;   // default number of fruitless polls before a tile gives up (seconds; never reached)
constexpr uint32_t LOOK_BATCH = 8;               // earlier tiles looked at per round trip (registers: two per tile)
constexpr uint32_t ONESWEEP_SPREAD = 64;         // neighbouring workgroups of a pass work this many tile ranges apart
__host__ __device__ inline uint32_t onesweep_grid(uint32_t n_tiles) { return ((n_tiles + ONESWEEP_SPREAD - 1) / ONESWEEP_SPREAD) * ONESWEEP_SPREAD; }

struct TileSmem {
  uint64_t stage[TILE];
  uint32_t cnt[TILE_WAVES][256];
  uint32_t gdst[256];   // global destination of the first key of each digit, minus its local start
  uint32_t aux[8];
};

// One pass of the sort over one tile: stable scatter by the digit at `shift`.
//   ticket    [n_tasks] zero when the pass starts.  A workgroup is sent to a task by its number (spread so that
//             workgroups that start together work on different tasks: a task's tiles depend on one another, the tasks
//             do not), and takes the task's next tile from the task's counter.  So every tile a tile waits for was
//             taken earlier, by a workgroup that is already running: the waits always end.  Launch
//             onesweep_grid(n_tiles) workgroups.
//   bases     k_digit_bases' output; `pass` names the digit's row in it.
//   look      [n_tiles][256] words, zero (LOOK_EMPTY) when the pass starts.
// A tile that has polled a word spin_limit times in vain sets ERR_WAIT, publishes zeros and leaves without writing; tiles
// that see ERR_WAIT leave too, and no key is ever written outside its task: the call then fails, nothing hangs.
__global__ void __launch_bounds__(TILE_THREADS) __attribute__((amdgpu_waves_per_eu(4, 8)))   // (two workgroups per compute unit)
k_onesweep_pass(const uint64_t* __restrict__ off, uint32_t n_tasks, const uint32_t* __restrict__ tile_prefix,
                const uint32_t* __restrict__ bases, int pass, int shift, uint32_t n_tiles, uint32_t* __restrict__ ticket,
                unsigned long long* __restrict__ look, const uint64_t* __restrict__ key_in, uint64_t* __restrict__ key_out,
                const int64_t* __restrict__ exec_in, int64_t* __restrict__ exec_out,
                const int64_t* __restrict__ gap_in, int64_t* __restrict__ gap_out, uint32_t spin_limit, Ctrl* ctrl) {
  extern __shared__ __align__(16) unsigned char tile_raw[];
  TileSmem& sm = *reinterpret_cast<TileSmem*>(tile_raw);
  const uint32_t tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const uint32_t per = (n_tiles + ONESWEEP_SPREAD - 1) / ONESWEEP_SPREAD;
  const uint32_t home = (blockIdx.x % ONESWEEP_SPREAD) * per + blockIdx.x / ONESWEEP_SPREAD;   // a tile of the task to work on
  if (home >= n_tiles) return;
  const uint32_t t = task_of_tile(tile_prefix, n_tasks, home);
  const uint32_t tp = tile_prefix[t];
  if (tid == 0) sm.aux[7] = atomicAdd(&ticket[t], 1u);
  __syncthreads();
  const uint32_t jl = sm.aux[7];   // (below the task's number of tiles: as many workgroups are sent to a task as it has tiles)
  const uint32_t j = tp + jl;
  const uint64_t task_start = off[t];
  const uint64_t start = task_start + static_cast<uint64_t>(jl) * TILE;
  const uint64_t end = off[t + 1];
  const uint32_t m = static_cast<uint32_t>(end - start < TILE ? end - start : TILE);

  for (uint32_t d = lane; d < 256; d += WAVE) sm.cnt[w][d] = 0;
  __builtin_amdgcn_wave_barrier();

  const uint32_t wave_base = w * (TILE_KPT * WAVE);
  uint64_t k[TILE_KPT];
  uint32_t rk[TILE_KPT];
#pragma unroll
  for (int r = 0; r < TILE_KPT; ++r) {
    const uint32_t pos = wave_base + r * WAVE + lane;
    k[r] = pos < m ? key_in[start + pos] : 0;
  }
#pragma unroll
  for (int r = 0; r < TILE_KPT; ++r) {
    const uint32_t pos = wave_base + r * WAVE + lane;
    rk[r] = wave_rank_digit(static_cast<uint32_t>(k[r] >> shift) & 0xffu, pos < m, sm.cnt[w]);
  }
  tile_digit_offsets<TILE_WAVES>(sm.cnt, sm.aux, sm.gdst);   // gdst[d] = this tile's count of digit d, for now
  if (tid < 256) {
    const uint32_t own = sm.gdst[tid];
    const uint32_t ls = sm.cnt[0][tid];  // wave 0's start of digit tid == the digit's local start
    unsigned long long* mine = look + static_cast<uint64_t>(j) * 256 + tid;
    unsigned long long before = 0;   // keys with this digit in the task's earlier tiles
    bool gave_up = false;
    if (jl > 0) {
      // (the words carry their whole message themselves, count and state in one: no ordering with other memory is needed)
      __hip_atomic_store(mine, LOOK_OWN | own, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      // The task's earlier tiles are looked at LOOK_BATCH at a time (independent loads, one round trip), nearest first:
      // own counts add up until a tile is met that already knows the count up to itself.
      uint32_t back = 1, polls = 0;
      bool done = false;
      while (!done && back <= jl) {
        const uint32_t n = jl - back + 1 < LOOK_BATCH ? jl - back + 1 : LOOK_BATCH;
        unsigned long long v[LOOK_BATCH];
#pragma unroll
        for (uint32_t i = 0; i < LOOK_BATCH; ++i)
          v[i] = i < n ? __hip_atomic_load(look + static_cast<uint64_t>(j - back - i) * 256 + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                       : LOOK_EMPTY;
        uint32_t used = 0;
#pragma unroll
        for (uint32_t i = 0; i < LOOK_BATCH; ++i) {
          if (!done && used == i && i < n) {
            const unsigned long long state = v[i] & ~LOOK_COUNT;
            if (state != LOOK_EMPTY) {
              before += v[i] & LOOK_COUNT;
              ++used;
              done = state == LOOK_UPTO;
            }
          }
        }
        back += used;
        if (used == 0) {   // the nearest tile not yet looked at has published nothing so far
          if (++polls >= spin_limit) { gave_up = true; break; }
          __builtin_amdgcn_s_sleep(1);
        }
      }
    }
    if (gave_up) {
      atomicOr(&ctrl->status, ERR_WAIT);
      before = 0;
    }
    __hip_atomic_store(mine, LOOK_UPTO | ((before + own) & LOOK_COUNT), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t rel = bases[static_cast<uint64_t>(tp) * DIGIT_WORDS_PER_TILE + pass * 256 + tid] + static_cast<uint32_t>(before);
    sm.gdst[tid] = static_cast<uint32_t>(task_start) + rel - ls;  // modulo 2^32; positions fit 32 bits
  }
  uint32_t lpos[TILE_KPT];
#pragma unroll
  for (int r = 0; r < TILE_KPT; ++r) {
    const uint32_t pos = wave_base + r * WAVE + lane;
    lpos[r] = sm.cnt[w][static_cast<uint32_t>(k[r] >> shift) & 0xffu] + rk[r];
    if (pos < m) sm.stage[lpos[r]] = k[r];
  }
  __syncthreads();
  // (a thread of this workgroup that gave up set the bit before the barrier; a tile that does not see another tile's
  // bit yet writes inside its own task only)
  if (tid == 0) sm.aux[6] = __hip_atomic_load(&ctrl->status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & ERR_WAIT;
  __syncthreads();
  if (sm.aux[6]) return;   // (the same decision for the whole workgroup)
  const uint32_t lo32 = static_cast<uint32_t>(task_start), hi32 = static_cast<uint32_t>(end);
  // keys leave in sorted order: consecutive threads write consecutive addresses inside a digit run
  uint32_t dst[TILE_KPT];
#pragma unroll
  for (int r = 0; r < TILE_KPT; ++r) {
    const uint32_t i = tid + r * TILE_THREADS;
    dst[r] = hi32;
    if (i < m) {
      const uint64_t kk = sm.stage[i];
      dst[r] = sm.gdst[static_cast<uint32_t>(kk >> shift) & 0xffu] + i;
      if (dst[r] < lo32 || dst[r] >= hi32) dst[r] = hi32;   // (cannot happen; a place outside the task is never written)
      if (dst[r] != hi32) key_out[dst[r]] = kk;
    }
  }
  __syncthreads();
  // payload 1: execution time
#pragma unroll
  for (int r = 0; r < TILE_KPT; ++r) {
    const uint32_t pos = wave_base + r * WAVE + lane;
    if (pos < m) sm.stage[lpos[r]] = static_cast<uint64_t>(exec_in[start + pos]);
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < TILE_KPT; ++r) {
    const uint32_t i = tid + r * TILE_THREADS;
    if (i < m && dst[r] != hi32) exec_out[dst[r]] = static_cast<int64_t>(sm.stage[i]);
  }
  __syncthreads();
  // payload 2: idle time
#pragma unroll
  for (int r = 0; r < TILE_KPT; ++r) {
    const uint32_t pos = wave_base + r * WAVE + lane;
    if (pos < m) sm.stage[lpos[r]] = static_cast<uint64_t>(gap_in[start + pos]);
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < TILE_KPT; ++r) {
    const uint32_t i = tid + r * TILE_THREADS;
    if (i < m && dst[r] != hi32) gap_out[dst[r]] = static_cast<int64_t>(sm.stage[i]);
  }
}

}  // namespace fikit
