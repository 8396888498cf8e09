// Long tasks (more launches than one workgroup can hold): one most-significant-digit partition
// pass splits a task's launches by the top bits of the Kernel ID into buckets that do fit, and
// consecutive buckets are packed into units for the one-workgroup kernel.  Because the ID is a
// hash, the buckets are of similar size unless a single ID dominates the task; such a task (a
// bucket larger than a workgroup can hold) keeps the general sort-based path.
//
//   k_plan_msd     which tasks are long, how many tiles each has
//   k_hash_tiles   Kernel ID / execution time / idle time of every launch of a long task (Section
//                  3.2), plus the tile's histogram of top ID bits - the partition needs no extra
//                  read of the IDs
//   (scan)         flat exclusive scan of the histograms = scatter offsets
//   k_msd_units    bucket sizes -> units of at most FUSE_MID_MAX launches (or one larger bucket)
//   k_tile_scatter (sort_kernels.hip.h) the partition itself, LDS-staged
//   k_msd_task_rows / k_gather_units   row counts and final placement of the units' rows
#pragma once

#include "common.hip.h"
#include "profile_kernels.hip.h"
#include "sort_kernels.hip.h"
#include "task_kernels.hip.h"

namespace fikit {

constexpr uint32_t MSD_MAX_BITS = 8;
constexpr uint32_t MSD_SLOTS = 1u << MSD_MAX_BITS;   // unit slots reserved per long task

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
                           uint32_t* __restrict__ is_long, uint32_t* __restrict__ mtiles) {
  const uint64_t t = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (t > n_tasks) return;
  uint32_t l = 0, tiles = 0;
  if (t < n_tasks) {
    const uint64_t len = off[t + 1] - off[t];
    if (gflag[t] && len > FUSE_MAX) { l = 1; tiles = static_cast<uint32_t>((len + TILE - 1) / TILE); }
  }
  is_long[t] = l;
  mtiles[t] = tiles;
}

// One tile (TILE launches of one long task) per workgroup of 256 threads.
__global__ void __launch_bounds__(256)
k_hash_tiles(const fikit_launch* __restrict__ rec, const uint64_t* __restrict__ off, uint32_t n_tasks,
             const uint32_t* __restrict__ tile_prefix, uint64_t* __restrict__ ids, int64_t* __restrict__ e0,
             int64_t* __restrict__ g0, uint32_t* __restrict__ H, Ctrl* ctrl) {
  __shared__ uint32_t hist[256];
  const uint32_t j = blockIdx.x;
  const uint32_t t = task_of_tile(tile_prefix, n_tasks, j);
  const uint32_t tp = tile_prefix[t];
  const uint32_t tiles_t = tile_prefix[t + 1] - tp;
  const uint32_t jl = j - tp;
  const uint64_t task_start = off[t], task_end = off[t + 1];
  const uint64_t start = task_start + static_cast<uint64_t>(jl) * TILE;
  const uint32_t m = static_cast<uint32_t>(task_end - start < TILE ? task_end - start : TILE);
  const int shift = 64 - static_cast<int>(msd_bits(task_end - task_start));
  hist[threadIdx.x] = 0;
  __syncthreads();
  bool bad = false;
  for (uint32_t x = threadIdx.x; x < m; x += 256) {
    const uint64_t i = start + x;
    const uint4* p = reinterpret_cast<const uint4*>(rec + i);
    const uint4 a = p[0], b = p[1], c = p[2];
    const bool has_next = (i + 1 < task_end);
    int64_t next_start = 0;
    if (has_next) next_start = rec[i + 1].start_ns;
    const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    const uint64_t id = kernel_id_of(w);
    const int64_t st = static_cast<int64_t>((static_cast<uint64_t>(c.y) << 32) | c.x);
    const int64_t en = static_cast<int64_t>((static_cast<uint64_t>(c.w) << 32) | c.z);
    bad |= (en < st);
    int64_t gap = GAP_NONE;
    if (has_next) { gap = next_start - en; gap = gap < 0 ? 0 : gap; }
    ids[i] = id;
    e0[i] = en - st;
    g0[i] = gap;
    atomicAdd(&hist[static_cast<uint32_t>(id >> shift)], 1u);
  }
  if (bad) atomicOr(&ctrl->status, ERR_BAD_RECORD);
  __syncthreads();
  H[static_cast<uint64_t>(tp) * 256 + static_cast<uint64_t>(threadIdx.x) * tiles_t + jl] = hist[threadIdx.x];
}

// One wave per task: packs a long task's ID buckets into units.  A task with a bucket of more than
// FUSE_MAX launches keeps the general path (mflag 0); otherwise mflag 1 and gflag cleared.  The lanes
// fetch the bucket boundaries together, one lane packs (a short sequential pass over at most 256
// buckets in LDS), and the lanes together write the unused slots and the work lists.
__global__ void __launch_bounds__(WAVE)
k_msd_units(const uint64_t* __restrict__ off, uint32_t n_tasks, const uint32_t* __restrict__ long_prefix,
            const uint32_t* __restrict__ tile_prefix, const uint32_t* __restrict__ Hs,
            uint32_t* __restrict__ ustart, uint32_t* __restrict__ ulen, uint32_t* __restrict__ utask,
            uint32_t* __restrict__ udcount, uint32_t* __restrict__ mflag, uint32_t* __restrict__ gflag,
            uint32_t* __restrict__ lists, uint32_t list_stride, Ctrl* ctrl) {
  __shared__ uint32_t bstart[MSD_SLOTS + 1];   // where each bucket starts inside the task
  __shared__ uint32_t n_used, all_fit;
  const uint32_t t = blockIdx.x, lane = threadIdx.x;
  if (t >= n_tasks) return;
  if (lane == 0) mflag[t] = 0;
  if (long_prefix[t + 1] == long_prefix[t]) return;   // not a long task
  const uint32_t o = long_prefix[t];
  const uint64_t task_start = off[t], len = off[t + 1] - task_start;
  const uint32_t nb = 1u << msd_bits(len);
  const uint32_t tp = tile_prefix[t], tiles_t = tile_prefix[t + 1] - tp;
  const uint64_t hbase = static_cast<uint64_t>(tp) * 256;
  const uint32_t h0 = Hs[hbase];
  for (uint32_t d = lane; d <= nb; d += WAVE)
    bstart[d] = d < nb ? Hs[hbase + static_cast<uint64_t>(d) * tiles_t] - h0 : static_cast<uint32_t>(len);
  __syncthreads();
  const uint32_t u0 = o * MSD_SLOTS;
  if (lane == 0) {
    uint32_t u = u0;
    bool ok = true;
    uint32_t cur_start = 0, cur_len = 0;
    for (uint32_t d = 0; d < nb; ++d) {
      const uint32_t rel = bstart[d], sz = bstart[d + 1] - rel;
      if (sz > FUSE_MAX) ok = false;
      if (cur_len > 0 && cur_len + sz > FUSE_MID_MAX) {
        ustart[u] = static_cast<uint32_t>(task_start) + cur_start; ulen[u] = cur_len;
        ++u;
        cur_start = rel;
        cur_len = 0;
      }
      cur_len += sz;
    }
    if (cur_len > 0) {
      ustart[u] = static_cast<uint32_t>(task_start) + cur_start; ulen[u] = cur_len;
      ++u;
    }
    n_used = u - u0;
    all_fit = ok ? 1u : 0u;
    if (ok) {
      mflag[t] = 1;
      gflag[t] = 0;
      atomicAdd(reinterpret_cast<unsigned long long*>(&ctrl->n_general), ~0ull);   // one general task fewer
    }
  }
  __syncthreads();   // (also makes lane 0's unit entries visible to the other lanes)
  const uint32_t used = all_fit ? n_used : 0;
  for (uint32_t k = lane; k < MSD_SLOTS; k += WAVE) {
    const uint32_t u = u0 + k;
    utask[u] = t;
    udcount[u] = 0;
    if (k >= used) { ustart[u] = 0; ulen[u] = 0; continue; }
    // work lists of units by size class (see k_classify)
    const uint32_t l = ulen[u];
    if (l == 0) continue;
    const uint32_t c = l <= FUSE_SMALL_MAX ? 0u : (l <= FUSE_MID_MAX ? 1u : 2u);
    lists[static_cast<uint64_t>(c) * list_stride + atomicAdd(&ctrl->n_class[c], 1u)] = u;
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
