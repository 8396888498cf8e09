// Whole-task profiling in one workgroup, for tasks that are short and have few distinct Kernel
// IDs (the regime the paper describes: a service repeats the same kernels over and over).
//
// One workgroup reads a task's launch records once, and produces its rows without ever writing
// per-launch intermediates to memory:
//   1. Kernel ID (Section 3.2 "Identifying each kernel"), execution time K and idle time G of
//      every launch stay in registers; the IDs are also written out in launch order.  Because
//      a task keeps launching the same few kernels, the hash of an identity (32 bytes) is
//      computed once and remembered in LDS under a cheap tag; later launches with the same 32
//      bytes (compared in full) reuse it.
//   2. The task's set of unique IDs (S_UID, Section 3.2) is built in an LDS hash table, then
//      ranked so that rows come out in ascending ID order.
//   3. count / sum / min / max per ID (sum / count = SK_j, SG_j of Section 3.2) by LDS atomics.
//   4. Nearest-rank p50 / p95 per ID: a histogram over each ID's own range of values (on a scale that keeps
//      the leading bits of large values) tells which bin holds each wanted rank; the few samples of those
//      bins are listed and ranked by counting.  If some list would get long (many equal or clustered
//      samples), most-significant-digit radix selection does the task instead: per pass, every launch whose
//      value still agrees with the digits fixed so far for its ID adds one to that ID's digit histogram,
//      and one thread per (ID, percentile) walks it to the digit that holds the wanted rank.
//   5. (Only when a gap fill follows in the same call.)  Algorithm 1 predicts a launch's duration and the idle time
//      after it from its ID's row.  With every launch's row number still in a register and the rows' medians or
//      means in LDS, the workgroup writes those predictions per launch itself, so that the gap fill does not have
//      to read the Kernel IDs again and look each one up.
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
constexpr uint32_t FUSE_SMALL_MAX = 4096;    // tasks up to this many launches: 512-thread workgroup, 8 launches per thread
constexpr uint32_t FUSE_MID_MAX = 8192;      // up to this many: 512-thread workgroup, 16 launches per thread
constexpr uint32_t FUSE_MAX = 16384;         // tasks up to this many launches: one larger workgroup
constexpr int FUSE_S_THREADS = 512, FUSE_S_WPE = 6, FUSE_S_LB = 1;            // shape for tasks up to FUSE_SMALL_MAX
constexpr int FUSE_M_THREADS = 1024, FUSE_M_DMAX = 512, FUSE_M_HIST = 16384;  // shape for tasks up to FUSE_MAX
constexpr bool FUSE_M_ESTATS = true;
constexpr uint32_t UNIT_RUNS_MAX = 1024;     // most tiles a long task may have for its units to be gathered (one run per tile)

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

// Remembered kernel identities: the 32 identity bytes (two 16-byte halves), the Kernel ID they hash to
// and the slot that ID occupies in the ID table; `ready` holds the entry's tag once the rest is valid.
// One array per field: lanes that look at different entries then fall on different LDS banks
// (48-byte records would put every entry on one of only eight bank groups).
template <int HT>
struct Memo {
  uint4 wa[HT], wb[HT];
  uint64_t id[HT];
  uint32_t slot[HT];
  uint32_t ready[HT];
};

// With ESTATS the sums, minima and maxima are gathered while the records are being read (per slot
// of the ID table, since ranks are not known yet): the memory pipe is the busy one then, LDS is idle.
constexpr int PRIV_IDS = 16, PRIV_COPIES = 32, PRIV_N = PRIV_IDS * PRIV_COPIES;

template <int NT, int DMAX, int HIST_WORDS, bool ESTATS = false>
struct FusedSmem {
  static constexpr int HT = 2 * DMAX;
  static constexpr int HE = ESTATS ? HT : 1;
  uint64_t ht_key[HT];       // ID table (open addressing): the task's unique IDs
  uint32_t ht_cnt[HT];       // launches per ID
  uint16_t slot_rank[HT];    // slot -> rank of its ID among the task's IDs
  uint64_t rkey[DMAX];       // by rank: the ID
  uint32_t rcnt[DMAX];       //          number of execution-time samples
  uint32_t gcnt[DMAX];       //          number of idle-time samples
  uint4 pref[DMAX];          // radix selection: digits fixed so far (x exec p50, y exec p95, z gap p50, w gap p95)
  uint16_t kth[4][DMAX];     //                  rank still to find inside the current candidates
  uint8_t npass[2][DMAX];    //                  passes this ID's execution / idle times need (from their max)
  uint32_t memo_claim[HT];   // 0 = free, else the tag of the claiming identity
  union {
    Memo<HT> memo;           // phase 1
    struct { uint64_t ckey[DMAX]; uint32_t cslot[DMAX]; } tmp;   // phase 2
    struct {
      uint64_t esum[DMAX], gsum[DMAX]; uint32_t emin[DMAX], emax[DMAX], gmin[DMAX], gmax[DMAX];
      // With few IDs many lanes would hit the same few addresses; every ID then gets PRIV_COPIES
      // accumulators, one per lane modulo PRIV_COPIES (so that a wave's lanes fall on different banks),
      // which are merged afterwards.
      uint64_t p_esum[PRIV_N], p_gsum[PRIV_N];
      uint32_t p_emin[PRIV_N], p_emax[PRIV_N], p_gmin[PRIV_N], p_gmax[PRIV_N], p_gcnt[PRIV_N];
    } acc;  // phase 3
    uint32_t hist[HIST_WORDS];  // phase 4
  } u;
  uint32_t aux[NT / WAVE];
  uint32_t maxe, maxg;
  uint32_t ndist;
  uint32_t fallback;
  struct { uint64_t esum[HE], gsum[HE]; uint32_t emin[HE], emax[HE], gmin[HE], gmax[HE], nogap[HE]; } early;   // by slot
  uint16_t rslot[ESTATS ? DMAX : 1];   // rank -> slot
};

constexpr uint32_t NONE32 = 0xffffffffu;   // "no idle time after this launch" in the 32-bit value registers

// Where row j of a task is staged: the task's slice of stage_a, then its slice of stage_b.
__device__ __forceinline__ uint64_t* staged_row(int64_t* stage_a, int64_t* stage_b, uint64_t base, uint32_t m, uint32_t j) {
  const uint32_t cap1 = m >> 4;  // rows of 16 words that fit in m words
  return j < cap1 ? reinterpret_cast<uint64_t*>(stage_a + base) + static_cast<uint64_t>(j) * 16
                  : reinterpret_cast<uint64_t*>(stage_b + base) + static_cast<uint64_t>(j - cap1) * 16;
}

__device__ __forceinline__ uint32_t rotl32(uint32_t x, int k) { return (x << k) | (x >> (32 - k)); }

// Cheap, non-zero tag of the identity words; only used to find the remembered entry quickly.
__device__ __forceinline__ uint32_t identity_tag(const uint32_t (&w)[8]) {
  uint32_t t = w[0] ^ rotl32(w[1], 5) ^ rotl32(w[2], 11) ^ rotl32(w[3], 17) ^ rotl32(w[4], 23) ^ rotl32(w[5], 29) ^
               rotl32(w[6], 3) ^ rotl32(w[7], 13);
  t ^= t >> 15;
  t = t * 0x2c1b3c6du;
  t ^= t >> 13;
  return t | 1u;
}

// How the fast percentile path packs an (ID, array) pair's window into one word: the shift that turns a
// value's offset from the window's low end into a bin number, then the bins that hold the two wanted ranks.
constexpr int SEL_BINS_LOG2_MAX = 11;
constexpr uint32_t SEL_SHIFT_MASK = 0x3fu, SEL_LISTED = 0x40u, SEL_BIN_MASK = 0xfffu, SEL_NO_BIN = SEL_BIN_MASK;   // "no samples"
constexpr int SEL_B50_AT = 7, SEL_B95_AT = 19;
__device__ __forceinline__ uint32_t sel_shift(uint32_t y) { return y & SEL_SHIFT_MASK; }
__device__ __forceinline__ uint32_t sel_b50(uint32_t y) { return (y >> SEL_B50_AT) & SEL_BIN_MASK; }
__device__ __forceinline__ uint32_t sel_b95(uint32_t y) { return (y >> SEL_B95_AT) & SEL_BIN_MASK; }

// The scale on which the fast percentile path lays out its bins: the bit pattern of the value as a float, without
// its lowest 12 bits, i.e. the exponent and the leading 12 bits of the value.  Conversion rounds to nearest, which is
// monotone, so ranks found on the scale are ranks of the values; values below 2^SCALE_EXACT_BITS map one to one and
// come back exactly with value_of_scale.  Durations of one kernel spread over a range in proportion to their size
// (the workloads draw them lognormal): bins of equal width on this scale then hold similar numbers of samples, where
// bins of equal width in nanoseconds would crowd most samples into the lowest few.
constexpr uint32_t SCALE_EXACT_BITS = 12, SCALE_DROP = 12;
__device__ __forceinline__ uint32_t scale_of(uint32_t v) { return __float_as_uint(__uint2float_rn(v)) >> SCALE_DROP; }
__device__ __forceinline__ uint32_t value_of_scale(uint32_t t) { return static_cast<uint32_t>(__uint_as_float(t << SCALE_DROP)); }

// log2 of the number of bins the fast percentile path cuts an ID's value range into: about one bin
// per WINDOW_SAMPLES_PER_BIN samples (the bin that holds a wanted rank is ranked directly afterwards), at least 2,
// at most 2^max_log2.
constexpr uint32_t WINDOW_SAMPLES_PER_BIN = 1;
__device__ __forceinline__ uint32_t window_bins_log2(uint32_t count, uint32_t max_log2) {
  const uint32_t want = count / WINDOW_SAMPLES_PER_BIN;
  const uint32_t lg = want <= 2 ? 1u : 32u - __builtin_clz(want - 1);
  return lg < max_log2 ? lg : max_log2;
}

// Number of samples of list[0 .. n) that sort before sample x (value v): smaller ones, and equal ones
// that stand earlier in the list.  Four independent reads per step.
__device__ __forceinline__ uint32_t list_rank(const uint32_t* list, uint32_t n, uint32_t v, uint32_t x) {
  uint32_t rank = 0;
  for (uint32_t y = 0; y < n; y += 4) {
#pragma unroll
    for (uint32_t u = 0; u < 4; ++u) {
      const uint32_t yy = y + u;
      const uint32_t o = list[yy < n ? yy : n - 1];
      rank += (yy < n && (o < v || (o == v && yy < x))) ? 1u : 0u;
    }
  }
  return rank;
}

// Values are kept as 32-bit numbers in registers (a task with an execution or idle time of
// 2^32 - 1 ns or more takes the general path), KPT launches per thread.
struct FusedArgs {
  // whole tasks read from launch records
  const fikit_launch* rec;
  const uint64_t* off;
  const uint32_t* list;        // work list of this launch: task numbers / unit numbers ...
  const uint32_t* count;       // ... and its length (workgroups beyond it have nothing to do)
  uint32_t max_len;            // capacity of this kernel shape (launches)
  uint64_t* ids;               // receives the IDs in launch order
  int64_t* e0;                 // per-launch values handed to the general path when a task does not fit
  int64_t* g0;
  uint64_t* key0;              // ... with their IDs, in the same order
  // units: groups of consecutive ID buckets of a long task, whose launches lie bucket-ordered inside every tile
  const uint32_t* ustart;      // where the unit would start if the task were in bucket order: names its staging slice
  const uint32_t* ulen;
  const uint32_t* utask;
  const uint32_t* ubuckets;    // first bucket | (bucket after the last) << 16
  const uint32_t* tile_prefix; // first tile of every task
  const uint16_t* bound;       // bucket boundaries of the tiles (layout: see k_tile_partition)
  uint32_t tile_len;           // launches per tile
  const uint64_t* part_id;     // tile-ordered IDs
  const uint2* part_kg;        // tile-ordered (execution time, idle time or NONE32)
  uint32_t* mflag;             // cleared when a unit sends its task to the general path
  // both
  int64_t* stage_a;            // rows are staged in the task's / unit's own slice of these two arrays
  int64_t* stage_b;            // (for units they are also the source of exec and gap values)
  uint32_t* dcount;            // rows per task / per unit
  uint32_t* gflag;             // task takes the general path
  Ctrl* ctrl;
  // Predictions for a gap fill that follows (whole tasks only; pred_role null: none).  A task that is the
  // high-priority trace or the low-priority queue of some scenario gets the predicted value of every launch written
  // in the form the one-lane-per-scenario walk reads, and is marked in pred_done.
  const uint32_t* pred_role;   // per task: ROLE_HP | ROLE_LP
  uint32_t* pred_lp_e;         // per launch: predicted execution time (tasks used as queue)
  uint2* pred_hp_eg;           // per launch: predicted (execution time, idle time) (tasks used as trace)
  uint64_t* pred_lp_total;     // per task: sum of its launches' predicted execution times (queue)
  uint32_t* pred_done;         // per task: 1 once its predictions are written
  uint32_t predictor;          // a fikit_predictor
};

// Where the sums of step 1 keep the number of launches: a task of this kernel has at most 2^14 launches of less than
// 2^32 ns, so a sum stays below 2^46.
constexpr int EARLY_COUNT_AT = 46;
static_assert(FUSE_MAX <= (1u << (EARLY_COUNT_AT - 32)), "sums of execution times stay below the count's bits");

// Adds one launch's execution time and (if it has one) idle time to the sums, minima and maxima of ID-table slot s.
template <typename Smem>
__device__ __forceinline__ void early_stats(Smem& sm, uint32_t s, uint32_t e, uint32_t g) {
  // A minimum only falls and a maximum only rises: a value that does not pass what is read now cannot pass what is
  // there later, so most launches leave the four extremes alone.
  const uint32_t emin = __hip_atomic_load(&sm.early.emin[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  const uint32_t emax = __hip_atomic_load(&sm.early.emax[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  const uint32_t gmin = __hip_atomic_load(&sm.early.gmin[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  const uint32_t gmax = __hip_atomic_load(&sm.early.gmax[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  // the launch is counted in the same word as its execution time is summed in (EARLY_COUNT_AT)
  atomicAdd(reinterpret_cast<unsigned long long*>(&sm.early.esum[s]), static_cast<unsigned long long>(e) + (1ull << EARLY_COUNT_AT));
  if (e < emin) atomicMin(&sm.early.emin[s], e);
  if (e > emax) atomicMax(&sm.early.emax[s], e);
  if (g != NONE32) {
    atomicAdd(reinterpret_cast<unsigned long long*>(&sm.early.gsum[s]), static_cast<unsigned long long>(g));
    if (g < gmin) atomicMin(&sm.early.gmin[s], g);
    if (g > gmax) atomicMax(&sm.early.gmax[s], g);
  } else {
    atomicAdd(&sm.early.nogap[s], 1u);   // (the last launch of a run)
  }
}

template <int NT, int KPT, int DMAX, int HIST_WORDS, int LB, bool UNITS, int WPE, bool ESTATS = false>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(WPE, 8)))
k_task_fused(const FusedArgs A) {
  using Smem = FusedSmem<NT, DMAX, HIST_WORDS, ESTATS>;
  constexpr int HT = Smem::HT;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);
  Ctrl* ctrl = A.ctrl;
  if (ctrl->status & ERR_OFFSETS) return;
  if (blockIdx.x >= *A.count) return;
  const uint32_t unit = A.list[blockIdx.x];
  uint32_t t;          // owning task
  uint64_t base;       // first launch / first sorted position
  uint64_t len64;
  if (UNITS) {
    len64 = A.ulen[unit];
    base = A.ustart[unit];
    t = A.utask[unit];
  } else {
    t = unit;
    base = A.off[t];
    len64 = A.off[t + 1] - base;
  }
  if (len64 == 0 || len64 > A.max_len) return;   // (cannot happen for a listed item)
  const uint32_t m = static_cast<uint32_t>(len64);
  const fikit_launch* __restrict__ rec = A.rec;
  uint64_t* __restrict__ ids = A.ids;
  int64_t* __restrict__ e0 = A.e0;
  int64_t* __restrict__ g0 = A.g0;
  int64_t* __restrict__ stage_a = A.stage_a;
  int64_t* __restrict__ stage_b = A.stage_b;
  uint32_t* __restrict__ dcount = A.dcount;
  uint32_t* __restrict__ gflag = A.gflag;
  const uint32_t tid = threadIdx.x;

  for (uint32_t i = tid; i < HT; i += NT) {
    sm.ht_key[i] = HT_EMPTY; sm.ht_cnt[i] = 0; sm.memo_claim[i] = 0; sm.u.memo.ready[i] = 0;
    if (ESTATS) {
      sm.early.esum[i] = 0; sm.early.emin[i] = ~0u; sm.early.emax[i] = 0;
      sm.early.gsum[i] = 0; sm.early.gmin[i] = ~0u; sm.early.gmax[i] = 0; sm.early.nogap[i] = 0;
    }
  }
  if (tid == 0) { sm.ndist = 0; sm.fallback = 0; sm.maxe = 0; sm.maxg = 0; }
  __syncthreads();

  // ---- 1. read, identify, measure ------------------------------------------------------------
  uint32_t ev[KPT], gv[KPT];   // execution time, idle time (NONE32 for the task's last launch)
  uint32_t sl[KPT];            // ID-table slot, later the rank of the launch's ID
  uint32_t my_maxe = 0, my_maxg = 0;
  bool bad = false, wide = false;
  const uint32_t lane = lane_id();
#pragma unroll
  for (int r = 0; r < KPT; ++r) { ev[r] = 0; gv[r] = NONE32; sl[r] = 0; }
  if (UNITS) {
    // The unit's launches lie in one run per tile of its task: between the boundaries of its first bucket and of
    // the bucket after its last.  Run table in LDS (the space of the identity memo, which units do not use):
    // where each run starts in the tile-ordered arrays, and how many of the unit's launches precede it.
    uint32_t* run_at = reinterpret_cast<uint32_t*>(&sm.u);
    uint32_t* run_before = run_at + UNIT_RUNS_MAX;          // [tiles + 1]
    uint16_t* run_of = reinterpret_cast<uint16_t*>(run_before + UNIT_RUNS_MAX + 4);   // [m]: the run that holds each launch
    static_assert(sizeof(sm.u) >= (2 * UNIT_RUNS_MAX + 4) * 4 + 2 * NT * KPT, "run tables of a unit");
    static_assert(UNIT_RUNS_MAX <= 0x10000, "runs are numbered in 16 bits");
    const uint32_t ub = A.ubuckets[unit], d0 = ub & 0xffffu, d1 = ub >> 16;
    const uint32_t tp = A.tile_prefix[t], tiles_t = A.tile_prefix[t + 1] - tp;
    const uint64_t task_start = A.off[t];
    const uint16_t* b_lo = A.bound + static_cast<uint64_t>(tp) * (256 + 1) + static_cast<uint64_t>(d0) * tiles_t;
    const uint16_t* b_hi = A.bound + static_cast<uint64_t>(tp) * (256 + 1) + static_cast<uint64_t>(d1) * tiles_t;
    uint32_t carry = 0;
    for (uint32_t j0 = 0; j0 < tiles_t; j0 += NT) {   // (trip count is the same for every thread)
      const uint32_t j = j0 + tid;
      uint32_t lo = 0, c = 0;
      if (j < tiles_t) { lo = b_lo[j]; c = static_cast<uint32_t>(b_hi[j]) - lo; }
      uint32_t total;
      const uint32_t ex = block_excl_scan<NT>(c, sm.aux, total);
      if (j < tiles_t) {
        run_at[j] = static_cast<uint32_t>(task_start) + j * A.tile_len + lo;
        run_before[j] = carry + ex;
      }
      carry += total;
    }
    if (tid == 0) run_before[tiles_t] = carry;
    __syncthreads();
    if (carry != m) {   // (cannot happen: the unit's length is the sum of these runs)
      if (tid == 0) atomicOr(&ctrl->status, ERR_OFFSETS);
      return;
    }
    // every run writes its number over the launches it holds, so that a launch finds its run with one look
    for (uint32_t j = tid; j < tiles_t; j += NT) {
      const uint32_t hi = run_before[j + 1];
      for (uint32_t i = run_before[j]; i < hi; ++i) run_of[i] = static_cast<uint16_t>(j);
    }
    __syncthreads();
    // all of a thread's launches are located first and then read together, so that their loads are in flight at once
    uint32_t at[KPT];
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
      const uint32_t i = r * NT + tid;
      at[r] = 0;
      if (i < m) {
        const uint32_t j = run_of[i];
        at[r] = run_at[j] + (i - run_before[j]);
      }
    }
    uint64_t idq[KPT];
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
      idq[r] = 0;
      if (r * NT + tid < m) {
        idq[r] = A.part_id[at[r]];
        const uint2 kg = A.part_kg[at[r]];
        ev[r] = kg.x;
        gv[r] = kg.y;
      }
    }
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
      const uint32_t i = r * NT + tid;
      if (i < m) {
        const uint64_t id = idq[r];
        my_maxe = ev[r] > my_maxe ? ev[r] : my_maxe;
        if (gv[r] != NONE32) my_maxg = gv[r] > my_maxg ? gv[r] : my_maxg;
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
        if (!placed) atomicOr(&sm.fallback, 1u);
        if (ESTATS) early_stats(sm, h, ev[r], gv[r]);
        else atomicAdd(&sm.ht_cnt[h], 1u);
        sl[r] = h;
      }
    }
  } else {
  // LB rounds of loads are issued before the first of them is used, to keep more bytes in flight
#pragma unroll
  for (int r0 = 0; r0 < KPT; r0 += LB) {
    if (static_cast<uint32_t>(r0) * NT < m) {
      uint4 qa[LB], qb[LB], qc[LB];
      int64_t qn[LB];
      uint32_t qrun[LB], qnrun[LB];
#pragma unroll
      for (int u = 0; u < LB; ++u) {
        const uint32_t i = (r0 + u) * NT + tid;
        qa[u] = qb[u] = qc[u] = make_uint4(0, 0, 0, 0);
        qn[u] = 0;
        qrun[u] = 0; qnrun[u] = 1;
        if (i < m) {
          const uint4* p = reinterpret_cast<const uint4*>(rec + base + i);
          // A record is read once.  Its first 48 bytes are loaded with the hint that they will not be used again;
          // the load that touches its line last (the run) is an ordinary one: with every touch hinted the line is
          // fetched anew per touch and the kernel takes half as long again, with none it is a few percent slower.
          qa[u] = load_once(p); qb[u] = load_once(p + 1); qc[u] = load_once(p + 2);
          qrun[u] = rec[base + i].run;
          // the next launch is the next lane's; only the wave's last lane has to read it
          if (lane == WAVE - 1 && i + 1 < m) { qn[u] = rec[base + i + 1].start_ns; qnrun[u] = rec[base + i + 1].run; }
        }
      }
#pragma unroll
      for (int u = 0; u < LB; ++u) {
        const int r = r0 + u;
        const uint32_t i = r * NT + tid;
        const uint32_t nx_lo = from_next_lane(qc[u].x), nx_hi = from_next_lane(qc[u].y), nx_run = from_next_lane(qrun[u]);
        if (i < m) {
          const uint4 a = qa[u], b = qb[u], c = qc[u];
          const int64_t next_start = lane == WAVE - 1 ? qn[u] : static_cast<int64_t>((static_cast<uint64_t>(nx_hi) << 32) | nx_lo);
          const uint32_t next_run = lane == WAVE - 1 ? qnrun[u] : nx_run;
          const bool has_next = (i + 1 < m) && next_run == qrun[u];   // an idle time follows: same task, same run
          const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
          const int64_t start = static_cast<int64_t>((static_cast<uint64_t>(c.y) << 32) | c.x);
          const int64_t end = static_cast<int64_t>((static_cast<uint64_t>(c.w) << 32) | c.z);
          bad |= (end < start);
          const uint64_t e64 = static_cast<uint64_t>(end - start);
          wide |= (e64 >= NONE32);
          ev[r] = static_cast<uint32_t>(e64);
          my_maxe = ev[r] > my_maxe ? ev[r] : my_maxe;
          if (has_next) {
            const int64_t g = next_start - end;
            const uint64_t g64 = static_cast<uint64_t>(g < 0 ? 0 : g);
            wide |= (g64 >= NONE32);
            gv[r] = static_cast<uint32_t>(g64);
            my_maxg = gv[r] > my_maxg ? gv[r] : my_maxg;
          }
          // Has this identity been seen before?  Then its Kernel ID and slot are remembered.
          const uint32_t tag = identity_tag(w);
          uint32_t mh = tag & (HT - 1);
          uint64_t id = 0;
          uint32_t slot = 0;
          bool hit = false;
#pragma unroll 1
          for (int probe = 0; probe < 4; ++probe) {
            const uint32_t rd = __hip_atomic_load(&sm.u.memo.ready[mh], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (rd == tag) {
              const uint4 ma = sm.u.memo.wa[mh];
              const uint4 mb = sm.u.memo.wb[mh];
              if (ma.x == a.x && ma.y == a.y && ma.z == a.z && ma.w == a.w && mb.x == b.x && mb.y == b.y && mb.z == b.z &&
                  mb.w == b.w) {
                id = sm.u.memo.id[mh];
                slot = sm.u.memo.slot[mh];
                hit = true;
                break;
              }
            } else if (rd == 0 && __hip_atomic_load(&sm.memo_claim[mh], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == 0) {
              break;  // free entry: this identity has not been remembered
            }
            mh = (mh + 1) & (HT - 1);
          }
          if (!hit) {
            id = kernel_id_of(w);
            // ID table: open addressing, linear probing; the ID is already a hash
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
            if (!placed) atomicOr(&sm.fallback, 1u);
            slot = h;
            // remember it: claim a free entry near the tag's home, fill it, then publish the tag
            if (placed) {
              uint32_t ch = tag & (HT - 1);
#pragma unroll 1
              for (int probe = 0; probe < 4; ++probe) {
                const uint32_t old = atomicCAS(&sm.memo_claim[ch], 0u, tag);
                if (old == 0) {
                  sm.u.memo.wa[ch] = a;
                  sm.u.memo.wb[ch] = b;
                  sm.u.memo.id[ch] = id;
                  sm.u.memo.slot[ch] = slot;
                  __hip_atomic_store(&sm.u.memo.ready[ch], tag, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                  break;
                }
                if (old == tag) {
                  // same tag: the same identity is being (or has been) remembered by someone else, or a
                  // different identity shares the tag; either way leave this one out if it is the former
                  const uint32_t rd = __hip_atomic_load(&sm.u.memo.ready[ch], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
                  if (rd == 0) break;  // being written right now: do not wait for it
                  const uint4 ma = sm.u.memo.wa[ch];
                  const uint4 mb = sm.u.memo.wb[ch];
                  if (ma.x == a.x && ma.y == a.y && ma.z == a.z && ma.w == a.w && mb.x == b.x && mb.y == b.y &&
                      mb.z == b.z && mb.w == b.w)
                    break;
                }
                ch = (ch + 1) & (HT - 1);
              }
            }
          }
          ids[base + i] = id;
          if (ESTATS) early_stats(sm, slot, ev[r], gv[r]);
          else atomicAdd(&sm.ht_cnt[slot], 1u);
          sl[r] = slot;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  }
  if (bad) atomicOr(&ctrl->status, ERR_BAD_RECORD);
  if (wide) atomicOr(&sm.fallback, 1u);
  my_maxe = wave_max_u32(my_maxe);
  my_maxg = wave_max_u32(my_maxg);
  if (lane_id() == 0) { atomicMax(&sm.maxe, my_maxe); atomicMax(&sm.maxg, my_maxg); }
  __syncthreads();
  const uint32_t D = sm.ndist;
  if (sm.fallback || D > DMAX || D > 2 * (m >> 4)) {
    if (UNITS) {
      // the whole task goes to the general path (k_long_general_values hands its per-launch values over)
      if (tid == 0 && atomicExch(&A.mflag[t], 0u) == 1u) {
        gflag[t] = 1;
        atomicAdd(reinterpret_cast<unsigned long long*>(&ctrl->n_general), 1ull);
      }
      return;
    }
    // general path: hand over the per-launch values (recomputed at full width)
    // (every thread reads back the IDs it wrote itself)
    for (uint32_t i = tid; i < m; i += NT) {
      const fikit_launch* q = rec + base + i;
      const int64_t end = q->end_ns;
      e0[base + i] = end - q->start_ns;
      int64_t g = GAP_NONE;
      if (i + 1 < m && q[1].run == q->run) { g = q[1].start_ns - end; g = g < 0 ? 0 : g; }
      g0[base + i] = g;
      A.key0[base + i] = ids[base + i];
    }
    if (tid == 0) { gflag[t] = 1; atomicAdd(reinterpret_cast<unsigned long long*>(&ctrl->n_general), 1ull); }
    return;
  }

  // digit width of the radix selection: 16-bit counters, two per word, shared by 4 * D (ID, percentile) pairs
  int B = 31 - __builtin_clz(static_cast<uint32_t>(HIST_WORDS * 2) / (4 * D));
  B = B > 8 ? 8 : B;
  // the fast percentile path keeps one histogram per (ID, array) instead of four: its bins can be twice as fine
  // (as many bins as the 16-bit counters of 2 * D histograms leave room for, at most 2^SEL_BINS_LOG2_MAX; a row of
  // the histogram array holds one word, two bins, of every histogram and is 2 * D words long made odd)
  int B1 = 32 - __builtin_clz(static_cast<uint32_t>(HIST_WORDS) / ((2 * D) | 1u));
  B1 = B1 > SEL_BINS_LOG2_MAX ? SEL_BINS_LOG2_MAX : B1;

  // ---- 2. rank the distinct IDs --------------------------------------------------------------
  {
    uint32_t mine = 0;
    for (uint32_t s = tid; s < HT; s += NT) mine += (sm.ht_key[s] != HT_EMPTY);
    uint32_t total;
    uint32_t at = block_excl_scan<NT>(mine, sm.aux, total);   // (memo is dead after the barriers inside)
    for (uint32_t s = tid; s < HT; s += NT)
      if (sm.ht_key[s] != HT_EMPTY) { sm.u.tmp.ckey[at] = sm.ht_key[s]; sm.u.tmp.cslot[at] = s; ++at; }
    __syncthreads();
    for (uint32_t j = tid; j < D; j += NT) {
      const uint64_t k = sm.u.tmp.ckey[j];
      uint32_t rank = 0;
      for (uint32_t i = 0; i < D; ++i) rank += (sm.u.tmp.ckey[i] < k);
      const uint32_t s = sm.u.tmp.cslot[j];
      sm.slot_rank[s] = static_cast<uint16_t>(rank);
      if (ESTATS) sm.rslot[rank] = static_cast<uint16_t>(s);
      sm.rkey[rank] = k;
      sm.rcnt[rank] = ESTATS ? static_cast<uint32_t>(sm.early.esum[s] >> EARLY_COUNT_AT) : sm.ht_cnt[s];
    }
    __syncthreads();
  }
#pragma unroll
  for (int r = 0; r < KPT; ++r) sl[r] = sm.slot_rank[sl[r]];
  __syncthreads();  // tmp is dead from here on; acc reuses the space

  // ---- 3. count / sum / min / max per ID ------------------------------------------------------
  if (ESTATS) {
    // (gathered while reading, and so was the number of launches without an idle time)
  } else if (D <= static_cast<uint32_t>(PRIV_IDS)) {
    // few IDs: lane-private accumulators, merged afterwards
    const uint32_t np = D * PRIV_COPIES;
    for (uint32_t q = tid; q < np; q += NT) {
      sm.u.acc.p_esum[q] = 0; sm.u.acc.p_emin[q] = ~0u; sm.u.acc.p_emax[q] = 0;
      sm.u.acc.p_gsum[q] = 0; sm.u.acc.p_gmin[q] = ~0u; sm.u.acc.p_gmax[q] = 0;
      sm.u.acc.p_gcnt[q] = 0;
    }
    __syncthreads();
    const uint32_t copy = lane_id() & (PRIV_COPIES - 1);
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
      const uint32_t i = r * NT + tid;
      if (i < m) {
        const uint32_t q = sl[r] * PRIV_COPIES + copy;
        atomicAdd(reinterpret_cast<unsigned long long*>(&sm.u.acc.p_esum[q]), static_cast<unsigned long long>(ev[r]));
        atomicMin(&sm.u.acc.p_emin[q], ev[r]);
        atomicMax(&sm.u.acc.p_emax[q], ev[r]);
        if (gv[r] != NONE32) {
          atomicAdd(&sm.u.acc.p_gcnt[q], 1u);
          atomicAdd(reinterpret_cast<unsigned long long*>(&sm.u.acc.p_gsum[q]), static_cast<unsigned long long>(gv[r]));
          atomicMin(&sm.u.acc.p_gmin[q], gv[r]);
          atomicMax(&sm.u.acc.p_gmax[q], gv[r]);
        }
      }
    }
    __syncthreads();
    // merge: PRIV_COPIES consecutive lanes hold the copies of one ID (trip count is the same for all lanes of a wave)
    for (uint32_t q0 = 0; q0 < np; q0 += NT) {
      const uint32_t q = q0 + tid;
      const bool live = q < np;
      uint64_t es = live ? sm.u.acc.p_esum[q] : 0, gs = live ? sm.u.acc.p_gsum[q] : 0;
      uint32_t en = live ? sm.u.acc.p_emin[q] : ~0u, ex = live ? sm.u.acc.p_emax[q] : 0;
      uint32_t gn = live ? sm.u.acc.p_gmin[q] : ~0u, gx = live ? sm.u.acc.p_gmax[q] : 0, gc = live ? sm.u.acc.p_gcnt[q] : 0;
#pragma unroll
      for (int mk = PRIV_COPIES / 2; mk >= 1; mk >>= 1) {
        es += shfl_xor_u64(es, mk); gs += shfl_xor_u64(gs, mk);
        const uint32_t en2 = __shfl_xor(en, mk, WAVE), ex2 = __shfl_xor(ex, mk, WAVE);
        const uint32_t gn2 = __shfl_xor(gn, mk, WAVE), gx2 = __shfl_xor(gx, mk, WAVE);
        en = en2 < en ? en2 : en; ex = ex2 > ex ? ex2 : ex;
        gn = gn2 < gn ? gn2 : gn; gx = gx2 > gx ? gx2 : gx;
        gc += __shfl_xor(gc, mk, WAVE);
      }
      if (live && (q & (PRIV_COPIES - 1)) == 0) {
        const uint32_t j = q / PRIV_COPIES;
        sm.u.acc.esum[j] = es; sm.u.acc.emin[j] = en; sm.u.acc.emax[j] = ex;
        sm.u.acc.gsum[j] = gs; sm.u.acc.gmin[j] = gn; sm.u.acc.gmax[j] = gx;
        sm.gcnt[j] = gc;
      }
    }
  } else {
    for (uint32_t j = tid; j < D; j += NT) {
      sm.u.acc.esum[j] = 0; sm.u.acc.emin[j] = ~0u; sm.u.acc.emax[j] = 0;
      sm.u.acc.gsum[j] = 0; sm.u.acc.gmin[j] = ~0u; sm.u.acc.gmax[j] = 0;
      sm.gcnt[j] = 0;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
      const uint32_t i = r * NT + tid;
      if (i < m) {
        const uint32_t j = sl[r];
        atomicAdd(reinterpret_cast<unsigned long long*>(&sm.u.acc.esum[j]), static_cast<unsigned long long>(ev[r]));
        atomicMin(&sm.u.acc.emin[j], ev[r]);
        atomicMax(&sm.u.acc.emax[j], ev[r]);
        if (gv[r] != NONE32) {
          atomicAdd(&sm.gcnt[j], 1u);
          atomicAdd(reinterpret_cast<unsigned long long*>(&sm.u.acc.gsum[j]), static_cast<unsigned long long>(gv[r]));
          atomicMin(&sm.u.acc.gmin[j], gv[r]);
          atomicMax(&sm.u.acc.gmax[j], gv[r]);
        }
      }
    }
  }
  __syncthreads();
  // (predictions: a thread stages at most one row, DMAX <= NT, and keeps that ID's means for after the barrier)
  const bool emit = !UNITS && A.pred_role != nullptr;
  uint32_t mean_e = 0, mean_g = 0;
  for (uint32_t j = tid; j < D; j += NT) {
    uint64_t* row = staged_row(stage_a, stage_b, base, m, j);
    const uint32_t ec = sm.rcnt[j];
    uint32_t gc, emin, emax, gmin, gmax;
    uint64_t esum, gsum;
    if (ESTATS) {
      const uint32_t s = sm.rslot[j];
      gc = ec - sm.early.nogap[s];
      sm.gcnt[j] = gc;
      esum = sm.early.esum[s] & ((1ull << EARLY_COUNT_AT) - 1); emin = sm.early.emin[s]; emax = sm.early.emax[s];
      gsum = sm.early.gsum[s]; gmin = sm.early.gmin[s]; gmax = sm.early.gmax[s];
    } else {
      gc = sm.gcnt[j];
      esum = sm.u.acc.esum[j]; emin = sm.u.acc.emin[j]; emax = sm.u.acc.emax[j];
      gsum = sm.u.acc.gsum[j]; gmin = sm.u.acc.gmin[j]; gmax = sm.u.acc.gmax[j];
    }
    row[0] = sm.rkey[j];
    row[1] = t;
    row[2] = ec; row[3] = esum; row[4] = emin; row[5] = emax;
    row[8] = gc; row[9] = gsum;
    row[10] = gc ? gmin : 0; row[11] = gc ? gmax : 0;
    row[14] = 0; row[15] = 0;
    if (emit && A.predictor != FIKIT_PREDICT_P50) {
      mean_e = ec ? static_cast<uint32_t>(esum / ec) : 0u;
      mean_g = gc ? static_cast<uint32_t>(gsum / gc) : 0u;
    }
    sm.kth[0][j] = static_cast<uint16_t>(rank_index_u32(50, ec));
    sm.kth[1][j] = static_cast<uint16_t>(rank_index_u32(95, ec));
    sm.kth[2][j] = static_cast<uint16_t>(gc ? rank_index_u32(50, gc) : 0);
    sm.kth[3][j] = static_cast<uint16_t>(gc ? rank_index_u32(95, gc) : 0);
    sm.pref[j] = make_uint4(0, 0, 0, 0);
    const uint32_t mxe = emax, mxg = gc ? gmax : 0;
    {
      // window of the fast percentile path: the ID's own value range, cut into bins
      uint2* sel0 = reinterpret_cast<uint2*>(sm.ht_key);   // the ID table is dead by now
      const uint32_t lo_e = scale_of(emin), lo_g = scale_of(gc ? gmin : 0);
      const uint32_t re = scale_of(mxe) - lo_e, rg = scale_of(mxg) - lo_g;
      const uint32_t we = re ? 32 - __builtin_clz(re) : 0, wg = rg ? 32 - __builtin_clz(rg) : 0;
      const uint32_t be = window_bins_log2(ec, B1), bg = window_bins_log2(gc, B1);
      const uint32_t she = we > be ? we - be : 0, shg = wg > bg ? wg - bg : 0;
      // a bin that is one step wide on the part of the scale that is one to one is the answer;
      // otherwise the samples of the bin are listed and ranked
      const uint32_t exact = 1u << SCALE_EXACT_BITS;
      sel0[j] = make_uint2(lo_e, she | ((she || mxe >= exact) ? SEL_LISTED : 0u));
      sel0[D + j] = make_uint2(lo_g, shg | ((shg || mxg >= exact) ? SEL_LISTED : 0u));
    }
    sm.npass[0][j] = static_cast<uint8_t>(((mxe ? 32 - __builtin_clz(mxe) : 1) + B - 1) / B);
    sm.npass[1][j] = static_cast<uint8_t>(((mxg ? 32 - __builtin_clz(mxg) : 1) + B - 1) / B);
  }
  __syncthreads();  // acc is dead from here on; hist reuses the space
  static_assert(DMAX <= NT, "one staged row per thread at most");
  // predicted value per ID (by rank), in the space of the ranked IDs, which are in the rows by now
  uint32_t* pred_e = reinterpret_cast<uint32_t*>(sm.rkey);
  uint32_t* pred_g = pred_e + DMAX;
  const bool emit_p50 = emit && A.predictor == FIKIT_PREDICT_P50;
  if (emit && tid < D) { pred_e[tid] = mean_e; pred_g[tid] = mean_g; }
  // Writes the predictions of the task's launches (sl: rank of every launch's ID).  Called by all threads once the
  // percentiles are final.
  auto emit_predictions = [&]() {
    __syncthreads();
    const uint32_t rl = A.pred_role[t];
    if (rl & ROLE_LP) {
#pragma unroll
      for (int r = 0; r < KPT; ++r) {
        const uint32_t i = r * NT + tid;
        if (i < m) A.pred_lp_e[base + i] = pred_e[sl[r]];
      }
      if (tid < WAVE) {
        uint64_t total = 0;
        for (uint32_t j = tid; j < D; j += WAVE) total += static_cast<uint64_t>(sm.rcnt[j]) * pred_e[j];
        total = wave_sum_u64(total);
        if (tid == 0) A.pred_lp_total[t] = total;
      }
    }
    if (rl & ROLE_HP) {
#pragma unroll
      for (int r = 0; r < KPT; ++r) {
        const uint32_t i = r * NT + tid;
        if (i < m) { const uint32_t j = sl[r]; A.pred_hp_eg[base + i] = make_uint2(pred_e[j], pred_g[j]); }
      }
    }
    if (tid == 0 && rl != 0) A.pred_done[t] = 1u;
  };

  // ---- 4. nearest-rank percentiles ---------------------------------------------------------------
  // Fast way: one histogram pass over each ID's own value range [min, max] (2^B bins), which
  // tells in which bin the wanted rank lies; the few samples of that bin are then collected in
  // a short list and ranked directly.  If some bin is too crowded for that (many equal or
  // clustered samples), the general multi-pass radix selection below does the whole job instead.
  // Tables of earlier phases are dead by now and are reused:
  uint2* sel = reinterpret_cast<uint2*>(sm.ht_key);            // [2][DMAX]: x = window low end (on the scale), y = shift | listed | bin50 << 7 | bin95 << 19
  uint16_t* lcnt = reinterpret_cast<uint16_t*>(sm.ht_cnt);     // [2][2][DMAX]: list lengths (array, list A / B, ID)
  uint16_t* loff = reinterpret_cast<uint16_t*>(sm.memo_claim); // [2][2][DMAX]: list starts
  constexpr uint32_t LIST_MAX = 64;
  const uint32_t bins = 1u << B;
  const uint32_t P2 = 2 * D;   // (ID, array) pairs
  const uint32_t PS = P2 | 1u;  // row stride of the histogram array: odd, so that rows start on different LDS banks
  for (uint32_t i = tid; i < HIST_WORDS; i += NT) sm.u.hist[i] = 0;
  if (tid == 0) sm.fallback = 0;
  __syncthreads();
#pragma unroll
  for (int r = 0; r < KPT; ++r) {
    const uint32_t i = r * NT + tid;
    if (i < m) {
      uint32_t j = sl[r];
      asm volatile("" : "+v"(j));  // (an opaque copy: keeps the address arithmetic inside the loop, out of registers that live across it)
      const uint2 se = sel[j];
      const uint32_t de = (scale_of(ev[r]) - se.x) >> sel_shift(se.y);
      atomicAdd(&sm.u.hist[__umul24(de >> 1, PS) + j], (de & 1u) ? 0x10000u : 1u);
      if (gv[r] != NONE32) {
        const uint2 sg = sel[D + j];
        const uint32_t dg = (scale_of(gv[r]) - sg.x) >> sel_shift(sg.y);
        atomicAdd(&sm.u.hist[__umul24(dg >> 1, PS) + D + j], (dg & 1u) ? 0x10000u : 1u);
      }
    }
  }
  __syncthreads();
  {
    // 1, 2, 4 ... 64 lanes per (ID, array), as many as there are threads for: each sums its slice of the
    // pair's bins, a prefix sum over the slices tells which lane's slice holds each wanted rank, and
    // that lane finds the bin.
    const uint32_t per = static_cast<uint32_t>(NT) / P2;
    const uint32_t per_log2 = 31u - __builtin_clz(per | 1u);
    const uint32_t wg_log2 = per_log2 > 6u ? 6u : per_log2, WG = 1u << wg_log2;
    const uint32_t gl = tid & (WG - 1);
    for (uint32_t q0 = 0; q0 < P2; q0 += NT >> wg_log2) {   // (trip count is the same for all lanes of a wave)
      const uint32_t q = q0 + (tid >> wg_log2);
      const bool live = q < P2;
      const uint32_t arr = (live && q >= D) ? 1u : 0u, j = live ? q - arr * D : 0u;
      const uint32_t k50 = sm.kth[2 * arr][j], k95 = sm.kth[2 * arr + 1][j];
      const uint32_t cnt_all = arr ? sm.gcnt[j] : sm.rcnt[j];
      const uint32_t sy = live ? sel[q].y : 0u;
      const bool listed = (sy & SEL_LISTED) != 0;
      const uint32_t words = live ? (1u << window_bins_log2(cnt_all, B1)) >> 1 : 0u, wpl = ((words + WG - 1) >> wg_log2) | 1u;   // (odd: the lanes' slices start on different banks)
      const uint32_t w_lo = gl * wpl < words ? gl * wpl : words, w_hi = w_lo + wpl < words ? w_lo + wpl : words;
      uint32_t mine = 0, incl = 0;
      if (WG > 1) {
        for (uint32_t w = w_lo; w < w_hi; ++w) {
          const uint32_t pair = sm.u.hist[w * PS + q];
          mine += (pair & 0xffffu) + (pair >> 16);
        }
        // prefix over the group's lanes: a prefix over the wave, minus what precedes the group
        const uint32_t wave_incl = wave_incl_scan_u32(mine);
        const uint32_t first = lane_id() - gl;
        const uint32_t before_group = __shfl(wave_incl, first > 0 ? static_cast<int>(first) - 1 : 0, WAVE);
        incl = wave_incl - (first > 0 ? before_group : 0u);
      }
      // bins of this lane's slice that hold the wanted ranks (if any): bin number, rank inside it, its count
      uint32_t cum = incl - mine, bin50 = 0, n50 = 0, c50 = 0, bin95 = 0, n95 = 0, c95 = 0;
      bool has50 = false, has95 = false, same_bin = false;
      for (uint32_t w = w_lo; w < w_hi; ++w) {
        const uint32_t pair = sm.u.hist[w * PS + q];
        sm.u.hist[w * PS + q] = 0;
#pragma unroll
        for (uint32_t h = 0; h < 2; ++h) {
          const uint32_t c = h ? pair >> 16 : pair & 0xffffu;
          const bool f50 = k50 >= cum && k50 < cum + c, f95 = k95 >= cum && k95 < cum + c;
          if (f50) { has50 = true; bin50 = 2 * w + h; n50 = k50 - cum; c50 = c; }
          if (f95) { has95 = true; bin95 = 2 * w + h; n95 = k95 - cum; c95 = c; same_bin = k50 >= cum; }
          cum += c;
        }
      }
      if (live && cnt_all == 0) {
        if (gl == 0) {
          // no samples: both percentiles are 0, nothing to collect (SEL_NO_BIN never matches a bin number)
          sel[q].y = sy | (SEL_NO_BIN << SEL_B50_AT) | (SEL_NO_BIN << SEL_B95_AT);
          lcnt[(2 * arr) * DMAX + j] = 0;
          lcnt[(2 * arr + 1) * DMAX + j] = 0;
        }
      } else if (live) {
        // (bins that are the answer themselves: nothing to collect)
        if (has50) {
          const uint32_t la = listed ? c50 : 0u;
          atomicOr(&sel[q].y, bin50 << SEL_B50_AT);
          lcnt[(2 * arr) * DMAX + j] = static_cast<uint16_t>(la);
          if (listed) sm.kth[2 * arr][j] = static_cast<uint16_t>(n50);
          if (la > LIST_MAX) atomicOr(&sm.fallback, 1u);
        }
        if (has95) {
          // (the lower rank may lie in this bin too: then one list serves both)
          const uint32_t lb = (listed && !same_bin) ? c95 : 0u;
          atomicOr(&sel[q].y, bin95 << SEL_B95_AT);
          lcnt[(2 * arr + 1) * DMAX + j] = static_cast<uint16_t>(lb);
          if (listed) sm.kth[2 * arr + 1][j] = static_cast<uint16_t>(n95);
          if (lb > LIST_MAX) atomicOr(&sm.fallback, 1u);
        }
      }
    }
  }
  __syncthreads();
  const bool use_lists = (sm.fallback == 0);
  if (use_lists) {
    // list starts: exclusive scan of the 4 * D list lengths (order: array, list, ID)
    uint32_t carry = 0;
    for (uint32_t q0 = 0; q0 < 4 * D; q0 += NT) {
      const uint32_t q = q0 + tid;
      uint32_t c = 0, at = 0;
      if (q < 4 * D) { at = (q / D) * DMAX + (q % D); c = lcnt[at]; }
      uint32_t total;
      const uint32_t ex = block_excl_scan<NT>(c, sm.aux, total);
      if (q < 4 * D) loff[at] = static_cast<uint16_t>(carry + ex);
      carry += total;
    }
    // (4 * D lists of at most 64 samples: carry <= 4 * DMAX * 64 may exceed the space)
    const bool fits = carry <= static_cast<uint32_t>(HIST_WORDS);
    for (uint32_t j = tid; j < D; j += NT) {
      // pref's four words serve as the four list cursors of an ID; results go elsewhere until the end
      sm.pref[j] = make_uint4(0, 0, 0, 0);
    }
    __syncthreads();
    if (fits) {
      uint32_t* lists = sm.u.hist;
      uint32_t* cursor = reinterpret_cast<uint32_t*>(sm.pref);   // [ID][4]: exec A, exec B, gap A, gap B
#pragma unroll
      for (int r = 0; r < KPT; ++r) {
        const uint32_t i = r * NT + tid;
        if (i < m) {
          uint32_t j = sl[r];
          asm volatile("" : "+v"(j));  // (as above)
          const uint2 se = sel[j];
          if (se.y & SEL_LISTED) {
            const uint32_t de = (scale_of(ev[r]) - se.x) >> sel_shift(se.y), b50 = sel_b50(se.y), b95 = sel_b95(se.y);
            if (de == b50) lists[loff[j] + atomicAdd(&cursor[4 * j], 1u)] = ev[r];
            else if (de == b95) lists[loff[DMAX + j] + atomicAdd(&cursor[4 * j + 1], 1u)] = ev[r];
          }
          if (gv[r] != NONE32) {
            const uint2 sg = sel[D + j];
            if (sg.y & SEL_LISTED) {
              const uint32_t dg = (scale_of(gv[r]) - sg.x) >> sel_shift(sg.y), b50 = sel_b50(sg.y), b95 = sel_b95(sg.y);
              if (dg == b50) lists[loff[2 * DMAX + j] + atomicAdd(&cursor[4 * j + 2], 1u)] = gv[r];
              else if (dg == b95) lists[loff[3 * DMAX + j] + atomicAdd(&cursor[4 * j + 3], 1u)] = gv[r];
            }
          }
        }
      }
      __syncthreads();
      // eight lanes per (ID, array): every lane ranks some of the collected samples by counting how
      // many samples of the list precede them; the lane that finds the wanted rank writes the result
      constexpr uint32_t GS = 8;
      const uint32_t gl = tid % GS;
      for (uint32_t q = tid / GS; q < P2; q += NT / GS) {
        const uint32_t arr = q >= D ? 1u : 0u, j = q - arr * D;
        const uint2 se = sel[q];
        const uint32_t b50 = sel_b50(se.y), b95 = sel_b95(se.y);
        uint64_t* row = staged_row(stage_a, stage_b, base, m, j);
        if (b50 == SEL_NO_BIN || !(se.y & SEL_LISTED)) {   // (not listed: bins one value wide where the scale is one to one)
          if (gl == 0) {
            const uint32_t v50 = b50 == SEL_NO_BIN ? 0 : value_of_scale(se.x + b50);
            row[arr ? 12 : 6] = v50;
            if (emit_p50) (arr ? pred_g : pred_e)[j] = v50;
            row[arr ? 13 : 7] = b50 == SEL_NO_BIN ? 0 : value_of_scale(se.x + b95);
          }
          continue;
        }
        const uint32_t ca = lcnt[(2 * arr) * DMAX + j], cb = lcnt[(2 * arr + 1) * DMAX + j];
        const uint32_t k50 = sm.kth[2 * arr][j], k95 = sm.kth[2 * arr + 1][j];
        const uint32_t* la = lists + loff[(2 * arr) * DMAX + j];
        for (uint32_t x = gl; x < ca; x += GS) {
          const uint32_t v = la[x];
          const uint32_t rank = list_rank(la, ca, v, x);
          if (rank == k50) { row[arr ? 12 : 6] = v; if (emit_p50) (arr ? pred_g : pred_e)[j] = v; }
          if (cb == 0 && rank == k95) row[arr ? 13 : 7] = v;
        }
        if (cb) {
          const uint32_t* lb = lists + loff[(2 * arr + 1) * DMAX + j];
          for (uint32_t x = gl; x < cb; x += GS) {
            const uint32_t v = lb[x];
            const uint32_t rank = list_rank(lb, cb, v, x);
            if (rank == k95) row[arr ? 13 : 7] = v;
          }
        }
      }
      if (emit) emit_predictions();
      if (tid == 0) dcount[unit] = D;
      return;
    }
  }

  // ---- 4b. general way: multi-pass radix selection ------------------------------------------------
  __syncthreads();
  for (uint32_t j = tid; j < D; j += NT) {
    sm.pref[j] = make_uint4(0, 0, 0, 0);
    const uint32_t ec = sm.rcnt[j], gc = sm.gcnt[j];
    sm.kth[0][j] = static_cast<uint16_t>(rank_index_u32(50, ec));
    sm.kth[1][j] = static_cast<uint16_t>(rank_index_u32(95, ec));
    sm.kth[2][j] = static_cast<uint16_t>(gc ? rank_index_u32(50, gc) : 0);
    sm.kth[3][j] = static_cast<uint16_t>(gc ? rank_index_u32(95, gc) : 0);
  }
  __syncthreads();
  for (uint32_t i = tid; i < HIST_WORDS; i += NT) sm.u.hist[i] = 0;
  const uint32_t maxe = sm.maxe, maxg = sm.maxg;
  const int nbits_e = maxe ? 32 - __builtin_clz(maxe) : 1, nbits_g = maxg ? 32 - __builtin_clz(maxg) : 1;
  const uint32_t P = 4 * D;  // (ID, percentile) pairs
  const int passes_e = (nbits_e + B - 1) / B, passes_g = (nbits_g + B - 1) / B;
  const int passes = passes_e > passes_g ? passes_e : passes_g;
  __syncthreads();
  for (int p = passes - 1; p >= 0; --p) {
    const int shift = p * B;
    const int hi = shift + B;
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
      const uint32_t i = r * NT + tid;
      if (i < m) {
        uint32_t j = sl[r];
        asm volatile("" : "+v"(j));  // keep address arithmetic inside the pass
        const uint4 pf = sm.pref[j];
        // execution time: p50 (pair j) and p95 (pair D + j); one count serves both while their digits agree
        if (static_cast<uint32_t>(p) < sm.npass[0][j]) {
          const uint32_t v = ev[r];
          const bool m50 = hi >= 32 || ((v ^ pf.x) >> hi) == 0;
          const bool m95 = hi >= 32 || ((v ^ pf.y) >> hi) == 0;
          const uint32_t digit = (v >> shift) & (bins - 1);
          const uint32_t at = __umul24(digit >> 1, P) + j, inc = (digit & 1u) ? 0x10000u : 1u;
          if (m50) atomicAdd(&sm.u.hist[at], inc);
          if (m95 && pf.x != pf.y) atomicAdd(&sm.u.hist[at + D], inc);
        }
        if (gv[r] != NONE32 && static_cast<uint32_t>(p) < sm.npass[1][j]) {
          const uint32_t v = gv[r];
          const bool m50 = hi >= 32 || ((v ^ pf.z) >> hi) == 0;
          const bool m95 = hi >= 32 || ((v ^ pf.w) >> hi) == 0;
          const uint32_t digit = (v >> shift) & (bins - 1);
          const uint32_t at = __umul24(digit >> 1, P) + 2 * D + j, inc = (digit & 1u) ? 0x10000u : 1u;
          if (m50) atomicAdd(&sm.u.hist[at], inc);
          if (m95 && pf.z != pf.w) atomicAdd(&sm.u.hist[at + D], inc);
        }
      }
      __builtin_amdgcn_sched_barrier(0);  // keep the unrolled iterations apart: they would only cost registers
    }
    __syncthreads();
    // one thread per (ID, array) walks the digit counts to the bins that hold the wanted ranks
    for (uint32_t q = tid; q < 2 * D; q += NT) {
      const uint32_t arr = q >= D ? 1u : 0u, j = q - arr * D;
      if (static_cast<uint32_t>(p) < sm.npass[arr][j]) {
        const uint4 pf = sm.pref[j];
        const uint32_t p50 = arr ? pf.z : pf.x, p95 = arr ? pf.w : pf.y;
        const bool share = (p50 == p95);
        const uint32_t q50 = 2 * arr * D + j, q95 = q50 + D;
        const uint32_t k50 = sm.kth[2 * arr][j], k95 = sm.kth[2 * arr + 1][j];
        uint32_t cum = 0, d50 = 0, d95 = 0, n50 = 0, n95 = 0;
        bool f50 = false, f95 = false;
        for (uint32_t wd = 0; wd < (bins >> 1); ++wd) {
          const uint32_t pair = sm.u.hist[wd * P + q50];
          sm.u.hist[wd * P + q50] = 0;
          const uint32_t c0 = pair & 0xffffu, c1 = pair >> 16;
          if (!f50 && k50 < cum + c0) { f50 = true; d50 = 2 * wd; n50 = k50 - cum; }
          if (share && !f95 && k95 < cum + c0) { f95 = true; d95 = 2 * wd; n95 = k95 - cum; }
          cum += c0;
          if (!f50 && k50 < cum + c1) { f50 = true; d50 = 2 * wd + 1; n50 = k50 - cum; }
          if (share && !f95 && k95 < cum + c1) { f95 = true; d95 = 2 * wd + 1; n95 = k95 - cum; }
          cum += c1;
        }
        if (!share) {
          cum = 0;
          for (uint32_t wd = 0; wd < (bins >> 1); ++wd) {
            const uint32_t pair = sm.u.hist[wd * P + q95];
            sm.u.hist[wd * P + q95] = 0;
            const uint32_t c0 = pair & 0xffffu, c1 = pair >> 16;
            if (!f95 && k95 < cum + c0) { f95 = true; d95 = 2 * wd; n95 = k95 - cum; }
            cum += c0;
            if (!f95 && k95 < cum + c1) { f95 = true; d95 = 2 * wd + 1; n95 = k95 - cum; }
            cum += c1;
          }
        }
        if (f50) { sm.kth[2 * arr][j] = static_cast<uint16_t>(n50); if (arr) sm.pref[j].z = p50 | (d50 << shift); else sm.pref[j].x = p50 | (d50 << shift); }
        if (f95) { sm.kth[2 * arr + 1][j] = static_cast<uint16_t>(n95); if (arr) sm.pref[j].w = p95 | (d95 << shift); else sm.pref[j].y = p95 | (d95 << shift); }
      }
    }
    __syncthreads();
  }
  for (uint32_t j = tid; j < D; j += NT) {
    uint64_t* row = staged_row(stage_a, stage_b, base, m, j);
    const uint4 pf = sm.pref[j];
    row[6] = pf.x; row[7] = pf.y;
    row[12] = pf.z; row[13] = pf.w;
    if (emit_p50) { pred_e[j] = pf.x; pred_g[j] = pf.z; }
  }
  if (emit) emit_predictions();
  if (tid == 0) dcount[unit] = D;
}

// Moves a task's staged rows to their final place once the row offsets are known.
__global__ void __launch_bounds__(256)
k_gather_rows(const uint64_t* __restrict__ off, const uint32_t* __restrict__ row_off32, const uint32_t* __restrict__ gflag,
              const uint32_t* __restrict__ long_prefix, int have_long, const int64_t* __restrict__ stage_a,
              const int64_t* __restrict__ stage_b, uint32_t n_tasks, fikit_row* __restrict__ rows) {
  const uint32_t t = xcd_item(blockIdx.x, n_tasks);
  if (t >= n_tasks || gflag[t]) return;
  if (have_long && long_prefix[t + 1] != long_prefix[t]) return;   // a long task: its units are gathered separately
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
