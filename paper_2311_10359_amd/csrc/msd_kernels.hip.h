// Long tasks (more launches than one workgroup can hold): one pass over the launch records splits
// every tile of a task by the top bits of the Kernel ID, and the one-workgroup kernel then works on
// units of consecutive ID buckets, gathering each unit's launches from the tiles.  Because the ID is a
// hash, the buckets are of similar size unless a single ID dominates the task; such a task (a bucket
// larger than a workgroup can hold) keeps the general sort-based path.
//
//   k_plan_msd        which tasks are long, how many tiles each has
//   k_tile_partition  one tile per workgroup: Kernel ID / execution time / idle time of every launch
//                     (Section 3.2); the IDs leave in launch order (an output of the call), and the tile's
//                     launches leave again as (ID, execution time, idle time) triples ordered by bucket
//                     inside the tile's own index range, with the tile's table of bucket boundaries.
//                     Nothing depends on another tile: no counters, no waiting, one read of the records.
//   k_msd_units       bucket sizes of a task (summed over its tiles) -> units of at most FUSE_MID_MAX
//                     launches (or one larger bucket)
//   k_task_fused      (task_kernels.hip.h, unit form) reads a unit's launches as one run per tile
//   k_msd_task_rows / k_gather_units   row counts and final placement of the units' rows
//   k_long_general_values   per-launch values of long tasks that had to be left to the general path
#pragma once

#include "common.hip.h"
#include "profile_kernels.hip.h"
#include "sort_kernels.hip.h"
#include "task_kernels.hip.h"

namespace fikit {

constexpr uint32_t MSD_MAX_BITS = 8;
constexpr uint32_t MSD_SLOTS = 1u << MSD_MAX_BITS;   // unit slots reserved per long task
constexpr uint32_t PT_TILE = 4096;                   // launches per tile of the partition pass
constexpr int PT_THREADS = 512, PT_WAVES = PT_THREADS / WAVE, PT_KPT = PT_TILE / PT_THREADS;
constexpr int PT_LB = 2;                             // rounds of record loads in flight per lane
constexpr uint32_t PT_ROWS = MSD_SLOTS + 1;          // rows of a task's boundary table: bucket 0 .. 256 (= the tile's end)
static_assert(PT_TILE <= 0xffffu, "bucket boundaries inside a tile are stored in 16 bits");
static_assert(MSD_SLOTS * FUSE_MAX / PT_TILE <= UNIT_RUNS_MAX, "a unit's run table holds one run per tile of its task");

// Top ID bits used to partition a task of m launches: buckets of about FUSE_SMALL_MAX launches.
__host__ __device__ inline uint32_t msd_bits(uint64_t m) {
  const uint64_t want = (m + FUSE_SMALL_MAX - 1) / FUSE_SMALL_MAX;
  uint32_t b = 1;
  while ((1ull << b) < want && b < MSD_MAX_BITS) ++b;
  return b;
}

// is_long[t] = 1 for tasks that take this path, mtiles[t] = their number of tiles; both arrays have
// n_tasks + 1 entries (last 0) and are turned into prefix sums by the caller.
__global__ void k_plan_msd(const uint64_t* __restrict__ off, uint32_t n_tasks, const uint32_t* __restrict__ gflag,
                           uint32_t* __restrict__ is_long, uint32_t* __restrict__ mtiles, uint32_t* __restrict__ wflag) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (t > n_tasks) return;
  uint32_t l = 0, tiles = 0;
  if (t < n_tasks) {
    const uint64_t len = off[t + 1] - off[t];
    if (gflag[t] && len > FUSE_MAX) { l = 1; tiles = static_cast<uint32_t>((len + PT_TILE - 1) / PT_TILE); }
    wflag[t] = 0;
  }
  is_long[t] = l;
  mtiles[t] = tiles;
}

// Rank of this lane's key among the keys with the same `bits`-bit digit that the wave has seen so far (as
// wave_rank_digit, for digits narrower than eight bits).
__device__ __forceinline__ uint32_t wave_rank_bits(uint32_t digit, bool valid, uint32_t* cnt_w, uint32_t bits) {
  uint64_t same = ballot(valid);
  for (uint32_t b = 0; b < bits; ++b) {
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

struct PartSmem {
  uint64_t stage[PT_TILE];   // the tile's IDs in bucket order, then its values
  uint32_t cnt[PT_WAVES][256];
  uint32_t aux[8];
};

// One tile (PT_TILE launches of one long task) per workgroup.  The boundary table of a task is stored bucket-major,
// tile-minor (bound[(first tile of the task) * PT_ROWS + bucket * tiles + tile]) so that a unit reads the two
// boundaries it needs of all tiles as two contiguous vectors.  Execution and idle times travel as 32-bit numbers
// (idle time NONE32 = the task's last launch has none); a task with a value that does not fit is flagged and left
// to the general path.
__global__ void __launch_bounds__(PT_THREADS)
k_tile_partition(const fikit_launch* __restrict__ rec, const uint64_t* __restrict__ off, uint32_t n_tasks,
                 const uint32_t* __restrict__ tile_prefix, const uint32_t* __restrict__ long_prefix,
                 uint64_t* __restrict__ ids, uint64_t* __restrict__ part_id, uint2* __restrict__ part_kg,
                 uint16_t* __restrict__ bound, uint32_t* __restrict__ bucket_size, uint32_t* __restrict__ wflag, Ctrl* ctrl) {
  extern __shared__ __align__(16) unsigned char part_raw[];
  PartSmem& sm = *reinterpret_cast<PartSmem*>(part_raw);
  const uint32_t j = blockIdx.x;
  const uint32_t t = task_of_tile(tile_prefix, n_tasks, j);
  const uint32_t tp = tile_prefix[t];
  const uint32_t tiles_t = tile_prefix[t + 1] - tp;
  const uint32_t jl = j - tp;
  const uint64_t task_start = off[t], task_end = off[t + 1];
  const uint64_t start = task_start + static_cast<uint64_t>(jl) * PT_TILE;
  const uint32_t m = static_cast<uint32_t>(task_end - start < PT_TILE ? task_end - start : PT_TILE);
  const uint32_t bits = msd_bits(task_end - task_start);
  const int shift = 64 - static_cast<int>(bits);
  const uint32_t tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  for (uint32_t d = lane; d < 256; d += WAVE) sm.cnt[w][d] = 0;
  __builtin_amdgcn_wave_barrier();

  const uint32_t wave_base = w * (PT_KPT * WAVE);
  uint64_t idr[PT_KPT];
  uint2 kgr[PT_KPT];
  bool bad = false, wide = false;
#pragma unroll
  for (int r0 = 0; r0 < PT_KPT; r0 += PT_LB) {
    uint4 qa[PT_LB], qb[PT_LB], qc[PT_LB];
    int64_t qn[PT_LB];
    uint32_t qrun[PT_LB], qnrun[PT_LB];
#pragma unroll
    for (int u = 0; u < PT_LB; ++u) {
      const uint32_t pos = wave_base + (r0 + u) * WAVE + lane;
      qa[u] = qb[u] = qc[u] = make_uint4(0, 0, 0, 0);
      qn[u] = 0;
      qrun[u] = 0; qnrun[u] = 1;
      if (pos < m) {
        const uint64_t i = start + pos;
        const uint4* p = reinterpret_cast<const uint4*>(rec + i);
        qa[u] = p[0]; qb[u] = p[1]; qc[u] = p[2];
        qrun[u] = rec[i].run;
        // the next launch is the next lane's; only the wave's last lane has to read it
        if (lane == WAVE - 1 && i + 1 < task_end) { qn[u] = rec[i + 1].start_ns; qnrun[u] = rec[i + 1].run; }
      }
    }
#pragma unroll
    for (int u = 0; u < PT_LB; ++u) {
      const int r = r0 + u;
      const uint32_t pos = wave_base + r * WAVE + lane;
      const uint32_t nx_lo = from_next_lane(qc[u].x), nx_hi = from_next_lane(qc[u].y), nx_run = from_next_lane(qrun[u]);
      if (lane != WAVE - 1) { qn[u] = static_cast<int64_t>((static_cast<uint64_t>(nx_hi) << 32) | nx_lo); qnrun[u] = nx_run; }
      idr[r] = 0;
      kgr[r] = make_uint2(0, 0);
      if (pos < m) {
        const uint64_t i = start + pos;
        const uint4 a = qa[u], b = qb[u], c = qc[u];
        const uint32_t wd[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        const uint64_t id = kernel_id_of(wd);
        const int64_t st = static_cast<int64_t>((static_cast<uint64_t>(c.y) << 32) | c.x);
        const int64_t en = static_cast<int64_t>((static_cast<uint64_t>(c.w) << 32) | c.z);
        bad |= (en < st);
        const uint64_t e64 = static_cast<uint64_t>(en - st);
        wide |= (e64 >= NONE32);
        uint32_t g32 = NONE32;
        if (i + 1 < task_end && qnrun[u] == qrun[u]) {   // an idle time follows: same task, same run
          const int64_t g = qn[u] - en;
          const uint64_t g64 = static_cast<uint64_t>(g < 0 ? 0 : g);
          wide |= (g64 >= NONE32);
          g32 = static_cast<uint32_t>(g64);
        }
        ids[i] = id;
        idr[r] = id;
        kgr[r] = make_uint2(static_cast<uint32_t>(e64), g32);
      }
    }
  }
  if (bad) atomicOr(&ctrl->status, ERR_BAD_RECORD);
  if (ballot(wide) && lane == 0) atomicOr(&wflag[t], 1u);

  uint32_t rk[PT_KPT];
#pragma unroll
  for (int r = 0; r < PT_KPT; ++r) {
    const uint32_t pos = wave_base + r * WAVE + lane;
    rk[r] = wave_rank_bits(static_cast<uint32_t>(idr[r] >> shift), pos < m, sm.cnt[w], bits);
  }
  tile_digit_offsets<PT_WAVES>(sm.cnt, sm.aux, nullptr);
  // where each bucket starts inside the tile (buckets the task does not have start at the tile's end), and the
  // tile's share of the task's bucket sizes (integer adds: the totals do not depend on the order of the tiles)
  if (tid < 256) {
    const uint32_t first = sm.cnt[0][tid], next = tid < 255 ? sm.cnt[0][tid + 1] : m;
    bound[static_cast<uint64_t>(tp) * PT_ROWS + static_cast<uint64_t>(tid) * tiles_t + jl] = static_cast<uint16_t>(first);
    if (next > first) atomicAdd(&bucket_size[static_cast<uint64_t>(long_prefix[t]) * MSD_SLOTS + tid], next - first);
  }
  if (tid == 256) bound[static_cast<uint64_t>(tp) * PT_ROWS + static_cast<uint64_t>(MSD_SLOTS) * tiles_t + jl] = static_cast<uint16_t>(m);
  uint32_t at[PT_KPT];
#pragma unroll
  for (int r = 0; r < PT_KPT; ++r) {
    const uint32_t pos = wave_base + r * WAVE + lane;
    at[r] = sm.cnt[w][static_cast<uint32_t>(idr[r] >> shift)] + rk[r];
    if (pos < m) sm.stage[at[r]] = idr[r];
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < PT_KPT; ++r) {
    const uint32_t i = tid + r * PT_THREADS;
    if (i < m) part_id[start + i] = sm.stage[i];
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < PT_KPT; ++r) {
    const uint32_t pos = wave_base + r * WAVE + lane;
    if (pos < m) sm.stage[at[r]] = (static_cast<uint64_t>(kgr[r].y) << 32) | kgr[r].x;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < PT_KPT; ++r) {
    const uint32_t i = tid + r * PT_THREADS;
    if (i < m) {
      const uint64_t v = sm.stage[i];
      part_kg[start + i] = make_uint2(static_cast<uint32_t>(v), static_cast<uint32_t>(v >> 32));
    }
  }
}

// One workgroup per task: packs a long task's ID buckets into units.  A task with a bucket of more than
// FUSE_MAX launches, or with an execution or idle time that does not fit 32 bits, keeps the general path
// (mflag 0); otherwise mflag 1 and gflag cleared.  Thread d sums bucket d over the task's tiles, one thread
// packs (a short sequential pass over at most 256 buckets in LDS), and all threads together write the unit
// slots and the work lists.  bucket_size: the task's bucket sizes as the tiles added them up.
__global__ void __launch_bounds__(MSD_SLOTS)
k_msd_units(const uint64_t* __restrict__ off, uint32_t n_tasks, const uint32_t* __restrict__ long_prefix,
            const uint32_t* __restrict__ tile_prefix, const uint32_t* __restrict__ bucket_size, const uint32_t* __restrict__ wflag,
            uint32_t* __restrict__ ustart, uint32_t* __restrict__ ulen, uint32_t* __restrict__ utask,
            uint32_t* __restrict__ udcount, uint32_t* __restrict__ ubuckets, uint32_t* __restrict__ mflag,
            uint32_t* __restrict__ gflag, uint32_t* __restrict__ lists, uint32_t list_stride, Ctrl* ctrl) {
  __shared__ uint32_t bstart[MSD_SLOTS + 1];   // where each bucket starts inside the task (in bucket order)
  __shared__ uint32_t us[MSD_SLOTS], ul[MSD_SLOTS], ub[MSD_SLOTS];
  __shared__ uint32_t aux[8];
  __shared__ uint32_t n_used, all_fit;
  const uint32_t t = blockIdx.x, d = threadIdx.x;
  if (t >= n_tasks) return;
  if (d == 0) mflag[t] = 0;
  if (long_prefix[t + 1] == long_prefix[t]) return;   // not a long task
  const uint32_t o = long_prefix[t];
  const uint64_t task_start = off[t], len = off[t + 1] - task_start;
  const uint32_t nb = 1u << msd_bits(len);
  const uint32_t tiles_t = tile_prefix[t + 1] - tile_prefix[t];
  const uint32_t size = d < nb ? bucket_size[static_cast<uint64_t>(o) * MSD_SLOTS + d] : 0u;
  uint32_t total;
  const uint32_t before = block_excl_scan_256(size, aux, total);
  bstart[d] = before;
  if (d == 0) bstart[MSD_SLOTS] = total;
  __syncthreads();
  if (d == 0) {
    uint32_t u = 0;
    bool ok = total == len && tiles_t <= UNIT_RUNS_MAX && wflag[t] == 0;
    uint32_t cur_first = 0, cur_len = 0;
    for (uint32_t k = 0; k < nb; ++k) {
      const uint32_t sz = bstart[k + 1] - bstart[k];
      if (sz > FUSE_MAX) ok = false;
      if (cur_len > 0 && cur_len + sz > FUSE_MID_MAX) {
        us[u] = bstart[cur_first]; ul[u] = cur_len; ub[u] = cur_first | (k << 16);
        ++u;
        cur_first = k;
        cur_len = 0;
      }
      if (cur_len == 0) cur_first = k;
      cur_len += sz;
    }
    if (cur_len > 0) { us[u] = bstart[cur_first]; ul[u] = cur_len; ub[u] = cur_first | (nb << 16); ++u; }
    n_used = u;
    all_fit = ok ? 1u : 0u;
    if (ok) {
      mflag[t] = 1;
      gflag[t] = 0;
      atomicAdd(reinterpret_cast<unsigned long long*>(&ctrl->n_general), ~0ull);   // one general task fewer
    }
  }
  __syncthreads();
  const uint32_t used = all_fit ? n_used : 0;
  const uint32_t u = o * MSD_SLOTS + d;
  utask[u] = t;
  udcount[u] = 0;
  const bool live = d < used;
  const uint32_t l = live ? ul[d] : 0u;
  ustart[u] = live ? static_cast<uint32_t>(task_start) + us[d] : 0u;
  ulen[u] = l;
  ubuckets[u] = live ? ub[d] : 0u;
  // work lists of units by size class (see k_classify): one reservation per task and class (a counter that every
  // unit bumped on its own would serialise the whole launch on one address)
  const uint32_t c = !live ? 3u : (l <= FUSE_SMALL_MAX ? 0u : (l <= FUSE_MID_MAX ? 1u : 2u));
  __syncthreads();   // (aux is reused)
  for (uint32_t k = 0; k < 3; ++k) {
    uint32_t total;
    const uint32_t at = block_excl_scan_256(c == k ? 1u : 0u, aux, total);
    __shared__ uint32_t list_base;
    if (d == 0) list_base = total ? atomicAdd(&ctrl->n_class[k], total) : 0u;
    __syncthreads();
    if (c == k) lists[static_cast<uint64_t>(k) * list_stride + list_base + at] = u;
    __syncthreads();
  }
}

// Long tasks that the general path has to take after all (a bucket too large for a workgroup, too many
// distinct IDs in a unit, a value beyond 32 bits): the general path wants (ID, execution time, idle time)
// of every launch of the task, in any order, as 64-bit arrays.  They are unpacked from the tile-ordered
// triples; only a task with a value beyond 32 bits is measured again from its records.
__global__ void __launch_bounds__(256)
k_long_general_values(const fikit_launch* __restrict__ rec, const uint64_t* __restrict__ off, uint32_t n_tasks,
                      const uint32_t* __restrict__ tile_prefix, const uint32_t* __restrict__ gflag,
                      const uint32_t* __restrict__ wflag, const uint64_t* __restrict__ ids, uint64_t* __restrict__ key,
                      const uint2* __restrict__ part_kg, int64_t* __restrict__ e0, int64_t* __restrict__ g0) {
  const uint32_t j = blockIdx.x;
  const uint32_t t = task_of_tile(tile_prefix, n_tasks, j);
  if (!gflag[t]) return;
  const uint32_t jl = j - tile_prefix[t];
  const uint64_t task_end = off[t + 1];
  const uint64_t start = off[t] + static_cast<uint64_t>(jl) * PT_TILE;
  const uint32_t m = static_cast<uint32_t>(task_end - start < PT_TILE ? task_end - start : PT_TILE);
  const bool from_records = wflag[t] != 0;
  for (uint32_t x = threadIdx.x; x < m; x += 256) {
    const uint64_t i = start + x;
    if (from_records) {
      const int64_t en = rec[i].end_ns;
      int64_t gap = GAP_NONE;
      if (i + 1 < task_end && rec[i + 1].run == rec[i].run) { gap = rec[i + 1].start_ns - en; gap = gap < 0 ? 0 : gap; }
      key[i] = ids[i];
      e0[i] = en - rec[i].start_ns;
      g0[i] = gap;
    } else {
      const uint2 kg = part_kg[i];
      e0[i] = static_cast<int64_t>(kg.x);
      g0[i] = kg.y == NONE32 ? GAP_NONE : static_cast<int64_t>(kg.y);
    }
  }
}

// Row count of every long task that went through units, and each unit's first row inside its task.
__global__ void k_msd_task_rows(uint32_t n_tasks, const uint32_t* __restrict__ long_prefix, const uint32_t* __restrict__ mflag,
                                const uint32_t* __restrict__ udcount, uint32_t* __restrict__ urow, uint32_t* __restrict__ dcount) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (t >= n_tasks || long_prefix[t + 1] == long_prefix[t] || !mflag[t]) return;
  const uint32_t u0 = long_prefix[t] * MSD_SLOTS;
  uint32_t run = 0;
  for (uint32_t k = 0; k < MSD_SLOTS; ++k) { urow[u0 + k] = run; run += udcount[u0 + k]; }
  dcount[t] = run;
}

// Moves a unit's staged rows to their final place.
__global__ void __launch_bounds__(256)
k_gather_units(const uint32_t* __restrict__ ustart, const uint32_t* __restrict__ ulen, const uint32_t* __restrict__ utask,
               const uint32_t* __restrict__ udcount, const uint32_t* __restrict__ urow, const uint32_t* __restrict__ mflag,
               const uint32_t* __restrict__ row_off32, const int64_t* __restrict__ stage_a, const int64_t* __restrict__ stage_b,
               uint32_t n_units, fikit_row* __restrict__ rows) {
  const uint32_t u = xcd_item(blockIdx.x, n_units);
  if (u >= n_units) return;
  const uint32_t m = ulen[u];
  if (m == 0) return;
  const uint32_t t = utask[u];
  if (!mflag[t]) return;
  const uint32_t D = udcount[u];
  uint64_t* out = reinterpret_cast<uint64_t*>(rows + row_off32[t] + urow[u]);
  const uint64_t base = ustart[u];
  for (uint32_t x = threadIdx.x; x < D * 16; x += 256) {
    const uint32_t j = x >> 4, f = x & 15;
    out[x] = staged_row(const_cast<int64_t*>(stage_a), const_cast<int64_t*>(stage_b), base, m, j)[f];
  }
}

}  // namespace fikit
