// C ABI of the FIKIT trace-profiling and gap-fill library: argument checks, workspace
// carving and kernel sequencing.  All arithmetic of the method runs in the HIP kernels.
#include "fikit.h"

#include <hip/hip_runtime.h>

#include <mutex>

#include "common.hip.h"
#include "gapfill_kernels.hip.h"
#include "profile_kernels.hip.h"
#include "sort_kernels.hip.h"
#include "stats_kernels.hip.h"
#include "task_kernels.hip.h"
#include "msd_kernels.hip.h"
#include "prio_kernels.hip.h"
#include "pairing_kernels.hip.h"
#include "merge_kernels.hip.h"

namespace {

using namespace fikit;

constexpr uint64_t MAX_ELEMS = (1ull << 32) - (1ull << 24);
constexpr int WALK_GW = 64;   // lanes that share a scenario in the few-scenario walk

#define FIKIT_HIP(expr)                           \
  do {                                            \
    if ((expr) != hipSuccess) {                   \
      (void)hipGetLastError();                    \
      return FIKIT_HIP_ERROR;                     \
    }                                             \
  } while (0)

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }
inline uint32_t blocks_for(uint64_t items, uint32_t per_block) {
  uint64_t b = (items + per_block - 1) / per_block;
  return static_cast<uint32_t>(b == 0 ? 1 : b);
}

// Carves consecutive 256-byte aligned regions out of the workspace.
struct Carver {
  uint64_t at = 0;
  uint64_t take(uint64_t bytes) {
    const uint64_t here = at;
    at = align_up(at + bytes, 256);
    return here;
  }
};

struct ProfileLayout {
  uint64_t ctrl, k0, k1, k2, e0, e1, g0, g1, tiles, hist, sums, bits, word_prefix, gflag, dcount, total;
  uint64_t is_long, mtiles, mflag, wflag, bsize, units, lists;   // long-task partition path; work lists
  uint64_t max_tiles, max_ptiles, n_words, max_units;
};

ProfileLayout profile_layout(uint64_t n, uint32_t n_tasks) {
  ProfileLayout L;
  Carver c;
  L.n_words = (n + 63) / 64;
  uint64_t big_tasks = n / (static_cast<uint64_t>(LEAF) + 1);
  if (big_tasks > n_tasks) big_tasks = n_tasks;
  L.max_tiles = n / TILE + big_tasks;
  L.ctrl = c.take(256);
  L.k0 = c.take(n * 8);
  L.k1 = c.take(n * 8);      // long tasks: tile-ordered IDs; general path: keys (sorted in the end)
  L.k2 = c.take(n * 8 + 8);  // long tasks: tile-ordered values; general path: second key buffer, then segment starts
  L.e0 = c.take(n * 8);
  L.e1 = c.take(n * 8);      // also: first half of the staged rows of one-workgroup tasks
  L.g0 = c.take(n * 8);
  L.g1 = c.take(n * 8);      // also: second half of the staged rows
  L.tiles = c.take((static_cast<uint64_t>(n_tasks) + 1) * 4);
  uint64_t long_tasks = n / (static_cast<uint64_t>(FUSE_MAX) + 1);
  if (long_tasks > n_tasks) long_tasks = n_tasks;
  L.max_ptiles = n / PT_TILE + long_tasks;
  {
    // digit counts and look-back words of the sort passes; before them the bucket boundaries of the long tasks' tiles live here
    const uint64_t a = L.max_tiles * (DIGIT_WORDS_PER_TILE * 4 + 256 * 8), b = L.max_ptiles * PT_ROWS * 2;
    L.hist = c.take(a > b ? a : b);
  }
  uint64_t longest = L.max_tiles * 256;
  if (longest < static_cast<uint64_t>(n_tasks) + 1) longest = static_cast<uint64_t>(n_tasks) + 1;
  if (longest < L.n_words) longest = L.n_words;
  L.sums = c.take((longest / SCAN_TILE + 2) * 4);
  L.bits = c.take(L.n_words * 8);
  L.word_prefix = c.take(L.n_words * 4);
  L.gflag = c.take(static_cast<uint64_t>(n_tasks) * 4);
  L.dcount = c.take((static_cast<uint64_t>(n_tasks) + 1) * 4);
  L.is_long = c.take((static_cast<uint64_t>(n_tasks) + 1) * 4);
  L.mtiles = c.take((static_cast<uint64_t>(n_tasks) + 1) * 4);
  L.mflag = c.take(static_cast<uint64_t>(n_tasks) * 4);
  L.wflag = c.take(static_cast<uint64_t>(n_tasks) * 4);
  L.bsize = c.take(long_tasks * MSD_SLOTS * 4);   // bucket sizes of the long tasks
  L.max_units = long_tasks * MSD_SLOTS;
  L.units = c.take(L.max_units * 4 * 6);   // start, length, task, row count, first row, buckets
  {
    const uint64_t longest_list = L.max_units > n_tasks ? L.max_units : n_tasks;
    L.lists = c.take(longest_list * 4 * 3);
  }
  L.total = c.at;
  return L;
}

// In-place exclusive prefix sum of `count` 32-bit words; the grand total goes to *d_total (may be null).
int scan_u32(uint32_t* d_data, uint64_t count, uint32_t* d_sums, uint64_t* d_total, hipStream_t st) {
  const uint32_t nb = blocks_for(count, SCAN_TILE);
  hipLaunchKernelGGL(k_scan_reduce, dim3(nb), dim3(SCAN_BLOCK), 0, st, d_data, count, d_sums);
  hipLaunchKernelGGL(k_scan_spine, dim3(1), dim3(SCAN_BLOCK), 0, st, d_sums, static_cast<uint64_t>(nb), d_total);
  hipLaunchKernelGGL(k_scan_apply, dim3(nb), dim3(SCAN_BLOCK), 0, st, d_data, count, d_sums);
  FIKIT_HIP(hipGetLastError());
  return FIKIT_OK;
}

// ---- optional per-kernel timing (fikit_trace_*) ---------------------------------------------
// When enabled, every launch site records a HIP event on the caller's stream; at the end of
// the call the time between consecutive events is added to the entry of the launch that
// opened the interval.  Process-wide and not thread safe: a measurement aid, off by default.
constexpr int TRACE_MAX_MARKS = 192;
constexpr int TRACE_MAX_NAMES = 48;
struct TraceEntry { const char* name; double ms; int launches; };
bool g_trace_on = false;
uint32_t g_wait_limit = LOOK_SPIN_LIMIT;   // fikit_set_wait_limit
TraceEntry g_trace[TRACE_MAX_NAMES];
int g_trace_n = 0;

struct Tracer {
  hipStream_t st;
  hipEvent_t ev[TRACE_MAX_MARKS];
  const char* name[TRACE_MAX_MARKS];
  int n = 0;
  bool on;
  explicit Tracer(hipStream_t s, bool allowed = true) : st(s), on(allowed && g_trace_on) {}
  void mark(const char* what) {
    if (!on || n >= TRACE_MAX_MARKS) return;
    if (hipEventCreate(&ev[n]) != hipSuccess) { on = false; return; }
    (void)hipEventRecord(ev[n], st);
    name[n++] = what;
  }
  // Called once the stream has been synchronised (or on any early return).
  ~Tracer() {
    if (n == 0) return;
    if (n < TRACE_MAX_MARKS) mark("end");
    (void)hipStreamSynchronize(st);
    for (int i = 0; i + 1 < n; ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, ev[i], ev[i + 1]) != hipSuccess) { (void)hipGetLastError(); continue; }
      int k = 0;
      while (k < g_trace_n && g_trace[k].name != name[i]) ++k;
      if (k == g_trace_n) {
        if (g_trace_n == TRACE_MAX_NAMES) continue;
        g_trace[g_trace_n++] = TraceEntry{name[i], 0.0, 0};
      }
      g_trace[k].ms += ms;
      g_trace[k].launches += 1;
    }
    for (int i = 0; i < n; ++i) (void)hipEventDestroy(ev[i]);
  }
};

int status_from_bits(uint32_t bits) {
  if (bits & (ERR_OFFSETS | ERR_TASK_INDEX | ERR_GAP_OFFSETS | ERR_ACTUAL_GAP | ERR_LP_LIST | ERR_ROWS)) return FIKIT_INVALID_ARG;
  if (bits & ERR_BAD_RECORD) return FIKIT_BAD_RECORD;
  if (bits & ERR_UNKNOWN_ID) return FIKIT_UNKNOWN_ID;
  if (bits & ERR_LP_LIMIT) return FIKIT_UNSUPPORTED;
  if (bits & ERR_WAIT) return FIKIT_HIP_ERROR;
  return FIKIT_OK;
}

int read_ctrl(const Ctrl* d_ctrl, Ctrl* h, hipStream_t st) {
  FIKIT_HIP(hipMemcpyAsync(h, d_ctrl, sizeof(Ctrl), hipMemcpyDeviceToHost, st));
  FIKIT_HIP(hipStreamSynchronize(st));
  return FIKIT_OK;
}

template <int W>
int launch_prio_walk(hipStream_t st, const uint64_t* off, const uint32_t* hp_task, const uint64_t* lp_off,
                     const uint32_t* lp_task, const uint32_t* lp_prio, uint64_t n_scen, const uint64_t* gap_off,
                     const uint32_t* lp_e, const uint2* hp_eg, int64_t margin, int64_t min_gap, uint32_t* fill_count,
                     int64_t* filled_ns, uint64_t* placed, int64_t* placed_ns, uint32_t vec_ok, const Ctrl* ctrl) {
  FIKIT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_pf_walk<W>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                static_cast<int>(sizeof(PrioWalkSmem<W>))));
  hipLaunchKernelGGL(k_pf_walk<W>, dim3(blocks_for(n_scen * W, PW_THREADS)), dim3(PW_THREADS), sizeof(PrioWalkSmem<W>), st, off,
                     hp_task, lp_off, lp_task, lp_prio, n_scen, gap_off, lp_e, hp_eg, margin, min_gap, fill_count, filled_ns,
                     placed, placed_ns, vec_ok, ctrl);
  return FIKIT_OK;
}

}  // namespace

extern "C" {

int fikit_version(void) { return 1; }

void fikit_set_wait_limit(uint32_t polls) { g_wait_limit = polls ? polls : LOOK_SPIN_LIMIT; }

void fikit_trace_enable(int on) {
  g_trace_on = on != 0;
  g_trace_n = 0;
}

int fikit_trace_read(int index, const char** name, double* total_ms, int* launches) {
  if (index >= 0 && index < g_trace_n) {
    if (name) *name = g_trace[index].name;
    if (total_ms) *total_ms = g_trace[index].ms;
    if (launches) *launches = g_trace[index].launches;
  }
  return g_trace_n;
}

const char* fikit_status_string(int status) {
  switch (status) {
    case FIKIT_OK: return "ok";
    case FIKIT_INVALID_ARG: return "invalid argument";
    case FIKIT_WORKSPACE_TOO_SMALL: return "workspace too small";
    case FIKIT_ROW_CAPACITY: return "row capacity exceeded";
    case FIKIT_BAD_RECORD: return "record with end_ns < start_ns";
    case FIKIT_UNKNOWN_ID: return "launch ID missing from its task's profile";
    case FIKIT_HIP_ERROR: return "HIP runtime error";
    case FIKIT_UNSUPPORTED: return "beyond a stated limit of this call (list entries and launches of a scenario number 2^32 or more)";
    case FIKIT_TOO_LARGE: return "input larger than the built-in scratch buffer of fikit_gapfill_static";
    default: return "unknown status";
  }
}

size_t fikit_profile_workspace_bytes(uint64_t n_records, uint32_t n_tasks) {
  if (n_records >= MAX_ELEMS) return 0;
  return static_cast<size_t>(profile_layout(n_records, n_tasks).total);
}

}  // extern "C"

namespace {

// Where the one-workgroup kernels of the profile put the predictions for a gap fill that follows (see FusedArgs).
struct PredEmit {
  const uint32_t* role;
  uint32_t* lp_e;
  uint2* hp_eg;
  uint64_t* lp_total;
  uint32_t* done;
  uint32_t predictor;
};

// fikit_profile; with `emit` the kernels that hold a whole task in one workgroup also write the task's predictions.
int profile_run(const fikit_launch* d_records, uint64_t n_records, const uint64_t* d_task_offsets,
                uint32_t n_tasks, uint64_t* d_ids_out, fikit_row* d_rows_out, uint64_t row_capacity,
                uint64_t* d_task_row_offsets, uint64_t* h_n_rows, void* d_workspace, size_t workspace_bytes,
                void* hip_stream, const PredEmit* emit) {
  if (!h_n_rows) return FIKIT_INVALID_ARG;
  *h_n_rows = 0;
  if (!d_task_offsets || !d_task_row_offsets || !d_workspace) return FIKIT_INVALID_ARG;
  if (n_records >= MAX_ELEMS) return FIKIT_INVALID_ARG;
  if (n_records > 0 && (!d_records || n_tasks == 0)) return FIKIT_INVALID_ARG;
  if (row_capacity > 0 && !d_rows_out) return FIKIT_INVALID_ARG;
  if (!aligned(d_records, 16) || !aligned(d_task_offsets, 8) || !aligned(d_ids_out, 8) || !aligned(d_rows_out, 16) ||
      !aligned(d_task_row_offsets, 8) || !aligned(d_workspace, 256))
    return FIKIT_INVALID_ARG;
  const ProfileLayout L = profile_layout(n_records, n_tasks);
  if (workspace_bytes < L.total) return FIKIT_WORKSPACE_TOO_SMALL;

  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  unsigned char* ws = static_cast<unsigned char*>(d_workspace);
  Ctrl* ctrl = reinterpret_cast<Ctrl*>(ws + L.ctrl);
  const uint64_t n = n_records;
  uint64_t* ids = d_ids_out ? d_ids_out : reinterpret_cast<uint64_t*>(ws + L.k0);
  uint64_t* k1 = reinterpret_cast<uint64_t*>(ws + L.k1);
  uint64_t* k2 = reinterpret_cast<uint64_t*>(ws + L.k2);
  int64_t* e0 = reinterpret_cast<int64_t*>(ws + L.e0);
  int64_t* e1 = reinterpret_cast<int64_t*>(ws + L.e1);
  int64_t* g0 = reinterpret_cast<int64_t*>(ws + L.g0);
  int64_t* g1 = reinterpret_cast<int64_t*>(ws + L.g1);
  uint32_t* tiles = reinterpret_cast<uint32_t*>(ws + L.tiles);
  uint32_t* hist = reinterpret_cast<uint32_t*>(ws + L.hist);
  uint32_t* sums = reinterpret_cast<uint32_t*>(ws + L.sums);

  Tracer tr(st);
  tr.mark("setup");
  hipLaunchKernelGGL(k_clear_ctrl, dim3(1), dim3(64), 0, st, ctrl);
  hipLaunchKernelGGL(k_validate_offsets, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, d_task_offsets, n_tasks, n, ctrl);
  Ctrl h{};
  if (n == 0) {
    hipLaunchKernelGGL(k_fill_u32, dim3(blocks_for(2 * (static_cast<uint64_t>(n_tasks) + 1), 256)), dim3(256), 0, st,
                       reinterpret_cast<uint32_t*>(d_task_row_offsets), 2 * (static_cast<uint64_t>(n_tasks) + 1), 0u);
    FIKIT_HIP(hipGetLastError());
    if (int rc = read_ctrl(ctrl, &h, st)) return rc;
    return status_from_bits(h.status);
  }

  uint32_t* gflag = reinterpret_cast<uint32_t*>(ws + L.gflag);
  uint32_t* dcount = reinterpret_cast<uint32_t*>(ws + L.dcount);
  uint64_t* bits = reinterpret_cast<uint64_t*>(ws + L.bits);
  uint32_t* word_prefix = reinterpret_cast<uint32_t*>(ws + L.word_prefix);
  uint32_t* seg_start = reinterpret_cast<uint32_t*>(k2);

  // Short tasks with few distinct IDs: one workgroup each, records read once, rows staged.
  tr.mark("plan");
  uint32_t* lists = reinterpret_cast<uint32_t*>(ws + L.lists);
  hipLaunchKernelGGL(k_classify, dim3(blocks_for(static_cast<uint64_t>(n_tasks) + 1, 256)), dim3(256), 0, st, d_task_offsets,
                     n_tasks, FUSE_SMALL_MAX, FUSE_MID_MAX, FUSE_MAX, gflag, dcount, lists, ctrl);
  uint32_t* is_long = reinterpret_cast<uint32_t*>(ws + L.is_long);
  uint32_t* mtiles = reinterpret_cast<uint32_t*>(ws + L.mtiles);
  uint32_t* mflag = reinterpret_cast<uint32_t*>(ws + L.mflag);
  uint32_t* ustart = reinterpret_cast<uint32_t*>(ws + L.units);
  uint32_t* ulen = ustart + L.max_units;
  uint32_t* utask = ulen + L.max_units;
  uint32_t* udcount = utask + L.max_units;
  uint32_t* urow = udcount + L.max_units;
  uint32_t* ubuckets = urow + L.max_units;
  uint32_t* wflag = reinterpret_cast<uint32_t*>(ws + L.wflag);
  uint16_t* bound = reinterpret_cast<uint16_t*>(hist);
  uint2* part_kg = reinterpret_cast<uint2*>(k2);
  auto small = k_task_fused<FUSE_S_THREADS, FUSE_SMALL_MAX / FUSE_S_THREADS, 256, 7168, FUSE_S_LB, false, FUSE_S_WPE>;
  auto medium = k_task_fused<FUSE_M_THREADS, FUSE_MAX / FUSE_M_THREADS, FUSE_M_DMAX, FUSE_M_HIST, 2, false, 4, FUSE_M_ESTATS>;
  auto mid = k_task_fused<512, 16, 256, 7168, 2, false, 4>;
  auto small_u = k_task_fused<FUSE_S_THREADS, FUSE_SMALL_MAX / FUSE_S_THREADS, 256, 7168, 4, true, FUSE_S_WPE>;
  auto mid_u = k_task_fused<512, 16, 256, 7168, 4, true, 4>;
  auto medium_u = k_task_fused<FUSE_M_THREADS, FUSE_MAX / FUSE_M_THREADS, FUSE_M_DMAX, FUSE_M_HIST, 2, true, 4, FUSE_M_ESTATS>;
  constexpr size_t mid_lds = sizeof(FusedSmem<512, 256, 7168>);
  FIKIT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(mid), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(mid_lds)));
  FIKIT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(mid_u), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(mid_lds)));
  constexpr size_t small_lds = sizeof(FusedSmem<FUSE_S_THREADS, 256, 7168>),
                   medium_lds = sizeof(FusedSmem<FUSE_M_THREADS, FUSE_M_DMAX, FUSE_M_HIST, FUSE_M_ESTATS>);
  FIKIT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(small), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(small_lds)));
  FIKIT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(medium), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(medium_lds)));
  FIKIT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(small_u), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(small_lds)));
  FIKIT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(medium_u), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(medium_lds)));
  FusedArgs fa{};
  fa.rec = d_records; fa.off = d_task_offsets; fa.ids = ids; fa.e0 = e0; fa.g0 = g0; fa.key0 = k1;
  fa.stage_a = e1; fa.stage_b = g1; fa.dcount = dcount; fa.gflag = gflag; fa.ctrl = ctrl;
  if (emit) {
    fa.pred_role = emit->role; fa.pred_lp_e = emit->lp_e; fa.pred_hp_eg = emit->hp_eg; fa.pred_lp_total = emit->lp_total;
    fa.pred_done = emit->done; fa.predictor = emit->predictor;
  }
  {
    tr.mark("k_task_fused_small");
    fa.list = lists; fa.count = &ctrl->n_class[0]; fa.max_len = FUSE_SMALL_MAX;
    hipLaunchKernelGGL(small, dim3(n_tasks), dim3(FUSE_S_THREADS), small_lds, st, fa);
    tr.mark("k_task_fused_mid");
    fa.list = lists + n_tasks; fa.count = &ctrl->n_class[1]; fa.max_len = FUSE_MID_MAX;
    hipLaunchKernelGGL(mid, dim3(n_tasks), dim3(512), mid_lds, st, fa);
    tr.mark("k_task_fused_medium");
    fa.list = lists + 2 * static_cast<uint64_t>(n_tasks); fa.count = &ctrl->n_class[2]; fa.max_len = FUSE_MAX;
    hipLaunchKernelGGL(medium, dim3(n_tasks), dim3(FUSE_M_THREADS), medium_lds, st, fa);
    FIKIT_HIP(hipGetLastError());
  }
  tr.mark("host_sync");
  if (int rc = read_ctrl(ctrl, &h, st)) return rc;
  if (int rc = status_from_bits(h.status)) return rc;
  uint64_t n_units = 0;
  if (h.n_long > 0) {
    // Long tasks: one pass over the records orders every tile by the top ID bits (IDs out in launch order on
    // the way), then the one-workgroup kernel on units of buckets, which gathers its launches from the tiles.
    n_units = h.n_long * MSD_SLOTS;
    if (n_units > L.max_units) return FIKIT_HIP_ERROR;   // cannot happen: a long task has more than FUSE_MAX launches
    tr.mark("plan");
    hipLaunchKernelGGL(k_plan_msd, dim3(blocks_for(static_cast<uint64_t>(n_tasks) + 1, 256)), dim3(256), 0, st, d_task_offsets,
                       n_tasks, gflag, is_long, mtiles, wflag);
    if (int rc = scan_u32(is_long, static_cast<uint64_t>(n_tasks) + 1, sums, nullptr, st)) return rc;
    if (int rc = scan_u32(mtiles, static_cast<uint64_t>(n_tasks) + 1, sums, &ctrl->n_big_tiles, st)) return rc;
    tr.mark("host_sync");
    if (int rc = read_ctrl(ctrl, &h, st)) return rc;
    const uint64_t n_msd_tiles = h.n_big_tiles;
    if (n_msd_tiles == 0 || n_msd_tiles > L.max_ptiles) return FIKIT_HIP_ERROR;
    tr.mark("k_tile_partition");
    uint32_t* bucket_size = reinterpret_cast<uint32_t*>(ws + L.bsize);
    hipLaunchKernelGGL(k_fill_u32, dim3(blocks_for(h.n_long * MSD_SLOTS, 256)), dim3(256), 0, st, bucket_size, h.n_long * MSD_SLOTS, 0u);
    FIKIT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_tile_partition), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  static_cast<int>(sizeof(PartSmem))));
    hipLaunchKernelGGL(k_tile_partition, dim3(static_cast<uint32_t>(n_msd_tiles)), dim3(PT_THREADS), sizeof(PartSmem), st, d_records,
                       d_task_offsets, n_tasks, mtiles, is_long, ids, k1, part_kg, bound, bucket_size, wflag, ctrl);
    tr.mark("k_msd_units");
    hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, &ctrl->n_class[0], static_cast<uint64_t>(4), 0u);   // the lists are reused for units
    hipLaunchKernelGGL(k_msd_units, dim3(n_tasks), dim3(MSD_SLOTS), 0, st, d_task_offsets, n_tasks, is_long, mtiles, bucket_size, wflag,
                       ustart, ulen, utask, udcount, ubuckets, mflag, gflag, lists, static_cast<uint32_t>(n_units), ctrl);
    FusedArgs ua = fa;
    ua.pred_role = nullptr;   // (units are parts of tasks: their task's predictions are left to the gap fill)
    ua.ustart = ustart; ua.ulen = ulen; ua.utask = utask; ua.ubuckets = ubuckets; ua.tile_prefix = mtiles; ua.bound = bound;
    ua.tile_len = PT_TILE; ua.part_id = k1; ua.part_kg = part_kg; ua.mflag = mflag; ua.dcount = udcount;
    tr.mark("k_unit_fused_small");
    ua.list = lists; ua.count = &ctrl->n_class[0]; ua.max_len = FUSE_SMALL_MAX;
    hipLaunchKernelGGL(small_u, dim3(static_cast<uint32_t>(n_units)), dim3(FUSE_S_THREADS), small_lds, st, ua);
    tr.mark("k_unit_fused_mid");
    ua.list = lists + n_units; ua.count = &ctrl->n_class[1]; ua.max_len = FUSE_MID_MAX;
    hipLaunchKernelGGL(mid_u, dim3(static_cast<uint32_t>(n_units)), dim3(512), mid_lds, st, ua);
    tr.mark("k_unit_fused_medium");
    ua.list = lists + 2 * n_units; ua.count = &ctrl->n_class[2]; ua.max_len = FUSE_MAX;
    hipLaunchKernelGGL(medium_u, dim3(static_cast<uint32_t>(n_units)), dim3(FUSE_M_THREADS), medium_lds, st, ua);
    tr.mark("plan");
    hipLaunchKernelGGL(k_msd_task_rows, dim3(blocks_for(n_tasks, 64)), dim3(64), 0, st, n_tasks, is_long, mflag, udcount, urow, dcount);
    FIKIT_HIP(hipGetLastError());
    tr.mark("host_sync");
    if (int rc = read_ctrl(ctrl, &h, st)) return rc;
    if (int rc = status_from_bits(h.status)) return rc;
    if (h.n_general > 0) {
      tr.mark("k_long_general_values");
      hipLaunchKernelGGL(k_long_general_values, dim3(static_cast<uint32_t>(n_msd_tiles)), dim3(256), 0, st, d_records, d_task_offsets,
                         n_tasks, mtiles, gflag, wflag, ids, k1, part_kg, e0, g0);
    }
  }
  const bool any_general = h.n_general > 0;
  uint64_t n_heads = 0;

  if (any_general) {
    // General path: per-launch values are in memory (written by whichever kernel gave the task up);
    // sort by ID, find the segment heads.
    tr.mark("plan");
    hipLaunchKernelGGL(k_plan_tiles, dim3(blocks_for(static_cast<uint64_t>(n_tasks) + 1, 256)), dim3(256), 0, st,
                       d_task_offsets, n_tasks, gflag, tiles, ctrl);
    if (int rc = scan_u32(tiles, static_cast<uint64_t>(n_tasks) + 1, sums, &ctrl->n_big_tiles, st)) return rc;
    tr.mark("host_sync");
    if (int rc = read_ctrl(ctrl, &h, st)) return rc;
    if (int rc = status_from_bits(h.status)) return rc;
    const uint64_t n_big_tiles = h.n_big_tiles;
    if (n_big_tiles > L.max_tiles) return FIKIT_HIP_ERROR;  // cannot happen for valid offsets

    // keys start in k1 (in whatever order each task's triples were handed over) and end there sorted, payload in e0 / g0
    FIKIT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_leaf_sort), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  static_cast<int>(sizeof(LeafSmem))));
    tr.mark("k_leaf_sort");
    hipLaunchKernelGGL(k_leaf_sort, dim3(xcd_grid(n_tasks)), dim3(LEAF_THREADS), sizeof(LeafSmem), st, d_task_offsets, n_tasks, gflag, k1,
                       k1, e0, g0, ctrl);
    FIKIT_HIP(hipGetLastError());
    // Eight stable passes over the eight key bytes sort any keys.  Kernel IDs are hashes: a task's distinct IDs
    // almost always differ in their upper four bytes already, so four passes over those are tried first; the
    // head search below also notices keys that are still out of order, and then all eight passes are run on
    // what the four left (any order of the (key, values) triples is a valid start).
    FIKIT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_onesweep_pass), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  static_cast<int>(sizeof(TileSmem))));
    uint32_t* digit_counts = hist;                                                    // [tile][DIGIT_WORDS_PER_TILE]
    unsigned long long* look = reinterpret_cast<unsigned long long*>(ws + L.hist + L.max_tiles * DIGIT_WORDS_PER_TILE * 4);   // [tile][256]
    uint32_t* tickets = wflag;                                                        // one per task (the long-task path is done with this array)
    // Four passes over four key bytes, least significant first; each pass is one launch (see sort_kernels.hip.h).
    auto sort_passes = [&](int first_byte) -> int {
      uint64_t *kin = k1, *kout = k2;
      int64_t *ein = e0, *eout = e1, *gin = g0, *gout = g1;
      const uint32_t nt = static_cast<uint32_t>(n_big_tiles);
      tr.mark("k_digit_hist");
      hipLaunchKernelGGL(k_fill_u32, dim3(blocks_for(n_big_tiles * DIGIT_WORDS_PER_TILE, 1024)), dim3(256), 0, st, digit_counts,
                         n_big_tiles * DIGIT_WORDS_PER_TILE, 0u);
      hipLaunchKernelGGL(k_digit_hist, dim3(nt), dim3(256), 0, st, d_task_offsets, n_tasks, tiles, kin, first_byte, digit_counts);
      hipLaunchKernelGGL(k_digit_bases, dim3(n_tasks), dim3(256), 0, st, n_tasks, tiles, digit_counts);
      for (int pass = 0; pass < SORT_PASSES_PER_ROUND; ++pass) {
        tr.mark("k_onesweep_pass");
        hipLaunchKernelGGL(k_fill_u32, dim3(blocks_for(n_big_tiles * 512, 1024)), dim3(256), 0, st, reinterpret_cast<uint32_t*>(look),
                           n_big_tiles * 512, 0u);
        hipLaunchKernelGGL(k_fill_u32, dim3(blocks_for(n_tasks, 1024)), dim3(256), 0, st, tickets, static_cast<uint64_t>(n_tasks), 0u);
        hipLaunchKernelGGL(k_onesweep_pass, dim3(onesweep_grid(nt)), dim3(TILE_THREADS), sizeof(TileSmem), st, d_task_offsets, n_tasks,
                           tiles, digit_counts, pass, 8 * (first_byte + pass), nt, tickets, look, kin, kout, ein, eout, gin, gout, g_wait_limit, ctrl);
        FIKIT_HIP(hipGetLastError());
        uint64_t* tk = kin; kin = kout; kout = tk;
        int64_t* t = ein; ein = eout; eout = t;
        t = gin; gin = gout; gout = t;
      }
      return FIKIT_OK;   // (an even number of passes: keys and values end in the arrays they started in)
    };
    auto find_heads = [&]() -> int {
      tr.mark("heads");
      hipLaunchKernelGGL(k_head_bits, dim3(blocks_for(n, 256)), dim3(256), 0, st, k1, n, d_task_offsets, n_tasks, gflag, bits, ctrl);
      hipLaunchKernelGGL(k_popcount_words, dim3(blocks_for(L.n_words, 256)), dim3(256), 0, st, bits, L.n_words, word_prefix);
      if (int rc = scan_u32(word_prefix, L.n_words, sums, &ctrl->n_heads, st)) return rc;
      tr.mark("host_sync");
      if (int rc = read_ctrl(ctrl, &h, st)) return rc;
      return status_from_bits(h.status);   // (a wait of the sort that ran out)
    };
    if (n_big_tiles > 0)
      if (int rc = sort_passes(4)) return rc;
    if (int rc = find_heads()) return rc;
    if (h.wide) {
      hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, &ctrl->wide, static_cast<uint64_t>(1), 0u);
      if (int rc = sort_passes(0)) return rc;   // all eight bytes, least significant first
      if (int rc = sort_passes(4)) return rc;
      if (int rc = find_heads()) return rc;
      if (h.wide) return FIKIT_HIP_ERROR;   // cannot happen: eight passes sort
    }
    n_heads = h.n_heads;
    tr.mark("heads");
    hipLaunchKernelGGL(k_general_row_counts, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, d_task_offsets, n_tasks, gflag,
                       bits, word_prefix, n, static_cast<uint32_t>(n_heads), dcount);
  }

  // Row offsets of every task, and the total.
  tr.mark("row_offsets");
  if (int rc = scan_u32(dcount, static_cast<uint64_t>(n_tasks) + 1, sums, &ctrl->n_rows, st)) return rc;
  hipLaunchKernelGGL(k_widen_offsets, dim3(blocks_for(static_cast<uint64_t>(n_tasks) + 1, 256)), dim3(256), 0, st, dcount,
                     static_cast<uint64_t>(n_tasks) + 1, d_task_row_offsets);
  tr.mark("host_sync");
  if (int rc = read_ctrl(ctrl, &h, st)) return rc;
  const uint64_t n_rows = h.n_rows;
  *h_n_rows = n_rows;
  if (n_rows > row_capacity) return FIKIT_ROW_CAPACITY;

  tr.mark("k_gather_rows");
  hipLaunchKernelGGL(k_gather_rows, dim3(xcd_grid(n_tasks)), dim3(256), 0, st, d_task_offsets, dcount, gflag, is_long,
                     n_units > 0 ? 1 : 0, e1, g1, n_tasks, d_rows_out);
  if (n_units > 0)
    hipLaunchKernelGGL(k_gather_units, dim3(xcd_grid(static_cast<uint32_t>(n_units))), dim3(256), 0, st, ustart, ulen, utask,
                       udcount, urow, mflag, dcount, e1, g1, static_cast<uint32_t>(n_units), d_rows_out);
  if (any_general && n_heads > 0) {
    tr.mark("seg_starts");
    hipLaunchKernelGGL(k_seg_starts, dim3(blocks_for(L.n_words, 256)), dim3(256), 0, st, bits, word_prefix, L.n_words, n, n_heads,
                       seg_start);
    tr.mark("k_stats_small");
    hipLaunchKernelGGL(k_stats_small, dim3(blocks_for(n_heads, 4)), dim3(256), 0, st, seg_start, n_heads, d_task_offsets,
                       n_tasks, k1, e0, g0, bits, word_prefix, n, dcount, d_rows_out);
    // rows with long segments: by work list (the staging areas e1 / g1 are free once the rows are gathered)
    tr.mark("k_stats_lists");
    uint32_t* rlist = reinterpret_cast<uint32_t*>(e1);
    hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, &ctrl->n_class[0], static_cast<uint64_t>(2), 0u);
    hipLaunchKernelGGL(k_stats_lists, dim3(blocks_for(n_heads, 256)), dim3(256), 0, st, seg_start, n_heads, d_task_offsets,
                       n_tasks, rlist, ctrl);
    tr.mark("k_stats_big");
    const uint32_t big_grid = static_cast<uint32_t>(n_heads < 4096 ? n_heads : 4096);
    const uint32_t huge_grid = static_cast<uint32_t>(n_heads < 512 ? n_heads : 512);
    hipLaunchKernelGGL(k_stats_big<BIG_THREADS>, dim3(big_grid), dim3(BIG_THREADS), 0, st, seg_start, n_heads, d_task_offsets,
                       n_tasks, k1, e0, g0, bits, word_prefix, n, dcount, d_rows_out, rlist, &ctrl->n_class[0], 0u);
    tr.mark("k_stats_huge");
    hipLaunchKernelGGL(k_stats_big<HUGE_THREADS>, dim3(huge_grid), dim3(HUGE_THREADS), 0, st, seg_start, n_heads,
                       d_task_offsets, n_tasks, k1, e0, g0, bits, word_prefix, n, dcount, d_rows_out, rlist, &ctrl->n_class[1],
                       1u);
  }
  FIKIT_HIP(hipGetLastError());
  FIKIT_HIP(hipStreamSynchronize(st));
  return FIKIT_OK;
}

}  // namespace

extern "C" {

int fikit_profile(const fikit_launch* d_records, uint64_t n_records, const uint64_t* d_task_offsets,
                  uint32_t n_tasks, uint64_t* d_ids_out, fikit_row* d_rows_out, uint64_t row_capacity,
                  uint64_t* d_task_row_offsets, uint64_t* h_n_rows, void* d_workspace, size_t workspace_bytes,
                  void* hip_stream) {
  return profile_run(d_records, n_records, d_task_offsets, n_tasks, d_ids_out, d_rows_out, row_capacity, d_task_row_offsets,
                     h_n_rows, d_workspace, workspace_bytes, hip_stream, nullptr);
}

// The per-launch arrays of the gap fill are read in 64-byte pieces that may reach past the last launch.
constexpr uint64_t GF_PAD = 256;
// One lane per scenario pays off once there are about as many scenarios as the GPU has lanes to run at a time.
constexpr uint64_t GF_LANES_MIN_SCENARIOS = 4096;

}  // extern "C"

namespace {

constexpr uint64_t ws_align(uint64_t v) { return (v + 255) / 256 * 256; }

// Workspace of the gap fill: control block, task roles, two work lists, queue totals, three per-launch arrays.
constexpr uint64_t gapfill_ws_bytes(uint64_t n_ids, uint64_t n_tasks) {
  return 256 + ws_align(n_tasks * 4) + ws_align(n_tasks * 4 * 2) + ws_align(n_tasks * 8) + 2 * ws_align(n_ids * 8 + GF_PAD) +
         ws_align(n_ids * 8);
}

bool gapfill_params_ok(const fikit_gapfill_params* p) {
  return p && p->margin_ns >= 0 && p->min_gap_ns >= 0 && p->reserved == 0 && p->predictor >= FIKIT_PREDICT_P50 &&
         p->predictor <= FIKIT_PREDICT_MEAN;
}

// The gap fill in two parts: what has to come before the predictions (checks, task roles, work lists) and the rest.
enum GfPart { GF_ALL, GF_SETUP, GF_REST };

// Enqueues every kernel of the gap fill on `st`; `ws` holds gapfill_ws_bytes(n_ids, n_tasks) bytes whose first 64
// are the control block.  Nothing is read back and nothing is allocated here.
int gapfill_enqueue(hipStream_t st, Tracer& tr, const uint64_t* d_ids, uint64_t n_ids, const uint64_t* d_task_offsets,
                    uint32_t n_tasks, const fikit_row* d_rows, const uint64_t* d_task_row_offsets, const uint32_t* d_hp_task,
                    const uint32_t* d_lp_task, uint64_t n_scenarios, const fikit_gapfill_params* h_params,
                    const uint64_t* d_gap_offsets, uint64_t n_gaps, uint32_t* d_fill_count, int64_t* d_filled_ns,
                    int64_t* d_lp_completion_ns, uint64_t* d_lp_placed, unsigned char* ws, bool set_attributes,
                    GfPart part = GF_ALL, PredEmit* emit = nullptr) {
  Carver c;
  Ctrl* ctrl = reinterpret_cast<Ctrl*>(ws + c.take(256));
  uint32_t* role = reinterpret_cast<uint32_t*>(ws + c.take(static_cast<uint64_t>(n_tasks) * 4));
  uint32_t* glists = reinterpret_cast<uint32_t*>(ws + c.take(static_cast<uint64_t>(n_tasks) * 4 * 2));
  uint64_t* lp_total = reinterpret_cast<uint64_t*>(ws + c.take(static_cast<uint64_t>(n_tasks) * 8));
  int64_t* pe = reinterpret_cast<int64_t*>(ws + c.take(n_ids * 8 + GF_PAD));
  int64_t* pg = reinterpret_cast<int64_t*>(ws + c.take(n_ids * 8 + GF_PAD));
  int64_t* open = reinterpret_cast<int64_t*>(ws + c.take(n_ids * 8));
  // the 32-bit arrays of the one-lane-per-scenario kernels share the space of the 64-bit ones
  uint32_t* lp_e = reinterpret_cast<uint32_t*>(pe);
  uint2* hp_eg = reinterpret_cast<uint2*>(pg);

  const bool lanes = n_scenarios >= GF_LANES_MIN_SCENARIOS && n_gaps < MAX_ELEMS;
  if (emit) {   // (what a profile that runs between the two parts may fill in; only the lane kernels read this form)
    emit->role = lanes ? role : nullptr;
    emit->lp_e = lp_e; emit->hp_eg = hp_eg; emit->lp_total = lp_total; emit->predictor = static_cast<uint32_t>(h_params->predictor);
  }
  if (part != GF_REST) {
  tr.mark("gf_setup");
  hipLaunchKernelGGL(k_clear_ctrl, dim3(1), dim3(64), 0, st, ctrl);
  hipLaunchKernelGGL(k_fill_u32, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, role, static_cast<uint64_t>(n_tasks), 0u);
  hipLaunchKernelGGL(k_validate_offsets, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, d_task_offsets, n_tasks, n_ids, ctrl);
  hipLaunchKernelGGL(k_gf_scenarios, dim3(blocks_for(n_scenarios, 256)), dim3(256), 0, st, d_task_offsets, n_tasks, d_hp_task,
                     d_lp_task, n_scenarios, d_gap_offsets, n_gaps, role, ctrl);
  tr.mark("gf_lists");
  hipLaunchKernelGGL(k_gf_lists, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, d_task_offsets, n_tasks, role, 8192u, glists,
                     ctrl);
  FIKIT_HIP(hipGetLastError());
  }
  if (part == GF_SETUP) return FIKIT_OK;
  // Many scenarios: one lane per scenario on 32-bit predictions; the 64-bit kernels then only run if a
  // prediction did not fit (they check Ctrl::wide).  Few scenarios: the 64-bit kernels, a group of lanes each.
  if (lanes) {
    tr.mark("k_gf_predict32");
    hipLaunchKernelGGL(k_gf_predict32, dim3(n_tasks), dim3(PRED_THREADS), 0, st, d_ids, d_task_offsets, n_tasks, d_rows,
                       d_task_row_offsets, role, glists, static_cast<const int64_t*>(nullptr), lp_e, hp_eg, lp_total,
                       static_cast<uint32_t>(h_params->predictor), emit ? emit->done : static_cast<const uint32_t*>(nullptr), ctrl);
    tr.mark("k_gf_walk_lanes");
    if (set_attributes)
      FIKIT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_gf_walk_lanes<LW_PLAN>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(sizeof(LaneWalkSmem))));
    const uint32_t vec_ok = (aligned(d_fill_count, 16) && aligned(d_filled_ns, 16)) ? 1u : 0u;
    hipLaunchKernelGGL(k_gf_walk_lanes<LW_PLAN>, dim3(blocks_for(n_scenarios, LW_THREADS)), dim3(LW_THREADS), sizeof(LaneWalkSmem), st,
                       d_task_offsets, d_hp_task, d_lp_task, n_scenarios, d_gap_offsets, lp_e, hp_eg, lp_total,
                       h_params->margin_ns, h_params->min_gap_ns, d_fill_count, d_filled_ns, d_lp_completion_ns, d_lp_placed,
                       vec_ok, ctrl);
  }
  const uint32_t only_if_wide = lanes ? 1u : 0u;
  tr.mark("k_gf_predict");
  hipLaunchKernelGGL(k_gf_predict, dim3(n_tasks), dim3(PRED_THREADS), 0, st, d_ids, d_task_offsets, n_tasks, d_rows,
                     d_task_row_offsets, role, glists, pe, pg, open, only_if_wide, static_cast<uint32_t>(h_params->predictor), ctrl);
  tr.mark("k_gf_walk");
  hipLaunchKernelGGL((k_gf_walk<WALK_GW, true>), dim3(blocks_for(n_scenarios, 256 / WALK_GW)), dim3(256), 0, st, d_task_offsets, d_hp_task,
                     d_lp_task, n_scenarios, d_gap_offsets, pe, pg, open, h_params->margin_ns, h_params->min_gap_ns,
                     d_fill_count, d_filled_ns, d_lp_completion_ns, d_lp_placed, only_if_wide, ctrl);
  FIKIT_HIP(hipGetLastError());
  return FIKIT_OK;
}

}  // namespace

extern "C" {

size_t fikit_gapfill_workspace_bytes(uint64_t n_ids, uint32_t n_tasks, uint64_t n_scenarios) {
  (void)n_scenarios;
  if (n_ids >= MAX_ELEMS) return 0;
  return static_cast<size_t>(gapfill_ws_bytes(n_ids, n_tasks));
}

int fikit_gapfill(const uint64_t* d_ids, const uint64_t* d_task_offsets, uint32_t n_tasks, const fikit_row* d_rows,
                  const uint64_t* d_task_row_offsets, const uint32_t* d_hp_task, const uint32_t* d_lp_task,
                  uint64_t n_scenarios, const fikit_gapfill_params* h_params, const uint64_t* d_gap_offsets,
                  uint32_t* d_fill_count, int64_t* d_filled_ns, int64_t* d_lp_completion_ns, uint64_t* d_lp_placed,
                  void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  if (!gapfill_params_ok(h_params)) return FIKIT_INVALID_ARG;
  if (!d_task_offsets || !d_task_row_offsets || !d_workspace) return FIKIT_INVALID_ARG;
  if (n_scenarios >= MAX_ELEMS) return FIKIT_INVALID_ARG;
  if (n_scenarios > 0 && (!d_hp_task || !d_lp_task || !d_gap_offsets || !d_lp_completion_ns || !d_lp_placed || n_tasks == 0))
    return FIKIT_INVALID_ARG;
  if (!aligned(d_ids, 8) || !aligned(d_task_offsets, 8) || !aligned(d_rows, 16) || !aligned(d_task_row_offsets, 8) ||
      !aligned(d_hp_task, 4) || !aligned(d_lp_task, 4) || !aligned(d_gap_offsets, 8) || !aligned(d_fill_count, 4) ||
      !aligned(d_filled_ns, 8) || !aligned(d_lp_completion_ns, 8) || !aligned(d_lp_placed, 8) || !aligned(d_workspace, 256))
    return FIKIT_INVALID_ARG;
  if (n_scenarios == 0) return FIKIT_OK;

  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  // The element counts live on the device: total launches and total gaps.
  uint64_t n_ids = 0, n_gaps = 0;
  FIKIT_HIP(hipMemcpyAsync(&n_ids, d_task_offsets + n_tasks, 8, hipMemcpyDeviceToHost, st));
  FIKIT_HIP(hipMemcpyAsync(&n_gaps, d_gap_offsets + n_scenarios, 8, hipMemcpyDeviceToHost, st));
  FIKIT_HIP(hipStreamSynchronize(st));
  if (n_ids >= MAX_ELEMS) return FIKIT_INVALID_ARG;
  if (n_ids > 0 && (!d_ids || !d_rows)) return FIKIT_INVALID_ARG;
  if (n_gaps > 0 && (!d_fill_count || !d_filled_ns)) return FIKIT_INVALID_ARG;
  if (workspace_bytes < fikit_gapfill_workspace_bytes(n_ids, n_tasks, n_scenarios)) return FIKIT_WORKSPACE_TOO_SMALL;

  unsigned char* ws = static_cast<unsigned char*>(d_workspace);
  Tracer tr(st);
  if (int rc = gapfill_enqueue(st, tr, d_ids, n_ids, d_task_offsets, n_tasks, d_rows, d_task_row_offsets, d_hp_task, d_lp_task,
                               n_scenarios, h_params, d_gap_offsets, n_gaps, d_fill_count, d_filled_ns, d_lp_completion_ns,
                               d_lp_placed, ws, true))
    return rc;
  tr.mark("host_sync");
  Ctrl h{};
  if (int rc = read_ctrl(reinterpret_cast<const Ctrl*>(ws), &h, st)) return rc;
  return status_from_bits(h.status);
}

size_t fikit_profile_gapfill_workspace_bytes(uint64_t n_records, uint32_t n_tasks, uint64_t n_scenarios) {
  const size_t a = fikit_profile_workspace_bytes(n_records, n_tasks), b = fikit_gapfill_workspace_bytes(n_records, n_tasks, n_scenarios);
  if (a == 0 || b == 0) return 0;
  return static_cast<size_t>(ws_align(a) + ws_align(b) + ws_align(static_cast<uint64_t>(n_tasks) * 4));
}

int fikit_profile_gapfill(const fikit_launch* d_records, uint64_t n_records, const uint64_t* d_task_offsets, uint32_t n_tasks,
                          uint64_t* d_ids_out, fikit_row* d_rows_out, uint64_t row_capacity, uint64_t* d_task_row_offsets,
                          uint64_t* h_n_rows, const uint32_t* d_hp_task, const uint32_t* d_lp_task, uint64_t n_scenarios,
                          const fikit_gapfill_params* h_params, const uint64_t* d_gap_offsets, uint32_t* d_fill_count,
                          int64_t* d_filled_ns, int64_t* d_lp_completion_ns, uint64_t* d_lp_placed, void* d_workspace,
                          size_t workspace_bytes, void* hip_stream) {
  if (!h_n_rows) return FIKIT_INVALID_ARG;
  *h_n_rows = 0;
  if (!gapfill_params_ok(h_params)) return FIKIT_INVALID_ARG;
  if (!d_ids_out || !d_workspace || !d_task_offsets || n_records >= MAX_ELEMS || n_scenarios >= MAX_ELEMS) return FIKIT_INVALID_ARG;
  if (n_scenarios > 0 && (!d_hp_task || !d_lp_task || !d_gap_offsets || !d_lp_completion_ns || !d_lp_placed || n_tasks == 0))
    return FIKIT_INVALID_ARG;
  if (!aligned(d_hp_task, 4) || !aligned(d_lp_task, 4) || !aligned(d_gap_offsets, 8) || !aligned(d_fill_count, 4) ||
      !aligned(d_filled_ns, 8) || !aligned(d_lp_completion_ns, 8) || !aligned(d_lp_placed, 8) || !aligned(d_workspace, 256))
    return FIKIT_INVALID_ARG;
  const size_t need = fikit_profile_gapfill_workspace_bytes(n_records, n_tasks, n_scenarios);
  if (need == 0) return FIKIT_INVALID_ARG;
  if (workspace_bytes < need) return FIKIT_WORKSPACE_TOO_SMALL;
  unsigned char* ws = static_cast<unsigned char*>(d_workspace);
  const uint64_t prof_bytes = ws_align(fikit_profile_workspace_bytes(n_records, n_tasks));
  const uint64_t gf_bytes = ws_align(fikit_gapfill_workspace_bytes(n_records, n_tasks, n_scenarios));
  unsigned char* gf_ws = ws + prof_bytes;
  uint32_t* done = reinterpret_cast<uint32_t*>(gf_ws + gf_bytes);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (n_scenarios == 0)
    return fikit_profile(d_records, n_records, d_task_offsets, n_tasks, d_ids_out, d_rows_out, row_capacity, d_task_row_offsets,
                         h_n_rows, ws, prof_bytes, hip_stream);

  uint64_t n_gaps = 0;
  FIKIT_HIP(hipMemcpyAsync(&n_gaps, d_gap_offsets + n_scenarios, 8, hipMemcpyDeviceToHost, st));
  FIKIT_HIP(hipStreamSynchronize(st));
  if (n_gaps > 0 && (!d_fill_count || !d_filled_ns)) return FIKIT_INVALID_ARG;

  // 1. the gap fill's checks and task roles; 2. the profile, whose one-workgroup kernels also write the predictions
  // of the tasks that the scenarios use; 3. the predictions of the remaining tasks, and the fill.
  PredEmit emit{};
  emit.done = done;
  {
    Tracer tr(st);
    hipLaunchKernelGGL(k_fill_u32, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, done, static_cast<uint64_t>(n_tasks), 0u);
    if (int rc = gapfill_enqueue(st, tr, d_ids_out, n_records, d_task_offsets, n_tasks, d_rows_out, d_task_row_offsets, d_hp_task,
                                 d_lp_task, n_scenarios, h_params, d_gap_offsets, n_gaps, d_fill_count, d_filled_ns,
                                 d_lp_completion_ns, d_lp_placed, gf_ws, true, GF_SETUP, &emit))
      return rc;
  }
  if (int rc = profile_run(d_records, n_records, d_task_offsets, n_tasks, d_ids_out, d_rows_out, row_capacity, d_task_row_offsets,
                           h_n_rows, ws, prof_bytes, hip_stream, emit.role ? &emit : nullptr))
    return rc;
  Tracer tr(st);
  if (int rc = gapfill_enqueue(st, tr, d_ids_out, n_records, d_task_offsets, n_tasks, d_rows_out, d_task_row_offsets, d_hp_task,
                               d_lp_task, n_scenarios, h_params, d_gap_offsets, n_gaps, d_fill_count, d_filled_ns,
                               d_lp_completion_ns, d_lp_placed, gf_ws, true, GF_REST, &emit))
    return rc;
  tr.mark("host_sync");
  Ctrl h{};
  if (int rc = read_ctrl(reinterpret_cast<const Ctrl*>(gf_ws), &h, st)) return rc;
  return status_from_bits(h.status);
}

}  // extern "C"

namespace {

// ---- fikit_gapfill_static: the gap fill for callers that cannot allocate --------------------------------------
// Its workspace is a device array that is part of the library's code object.  Every GPU the library runs on holds
// its own copy at its own address; that address is looked up once per device, with the device current.
constexpr uint64_t STATIC_SCRATCH_BYTES = gapfill_ws_bytes(FIKIT_STATIC_MAX_IDS, FIKIT_STATIC_MAX_TASKS);
static_assert(STATIC_SCRATCH_BYTES <= (32ull << 20), "the built-in scratch buffer is meant to stay modest");
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int STATIC_MAX_DEVICES = 64;
std::mutex g_static_mutex;
unsigned char* g_static_scratch[STATIC_MAX_DEVICES] = {};

// Address of the current device's scratch array (set-up on the first call on that device).
int static_scratch_of_current_device(unsigned char** out) {
  int dev = -1;
  FIKIT_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) return FIKIT_HIP_ERROR;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (!g_static_scratch[dev]) {
    unsigned char* ptr = nullptr;
    FIKIT_HIP(hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)));
    if (!ptr) return FIKIT_HIP_ERROR;
    FIKIT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_gf_walk_lanes<LW_PLAN>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(sizeof(LaneWalkSmem))));
    g_static_scratch[dev] = ptr;
  }
  *out = g_static_scratch[dev];
  return FIKIT_OK;
}

// The status a finished call would return, from the error bits its kernels left.
__global__ void k_publish_status(const Ctrl* ctrl, int32_t* status_out) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const uint32_t bits = ctrl->status;
  int32_t st = FIKIT_OK;
  if (bits & (ERR_OFFSETS | ERR_TASK_INDEX | ERR_GAP_OFFSETS)) st = FIKIT_INVALID_ARG;
  else if (bits & ERR_UNKNOWN_ID) st = FIKIT_UNKNOWN_ID;
  *status_out = st;
}

}  // namespace

extern "C" {

int fikit_gapfill_static(const uint64_t* d_ids, uint64_t n_ids, const uint64_t* d_task_offsets, uint32_t n_tasks,
                         const fikit_row* d_rows, const uint64_t* d_task_row_offsets, const uint32_t* d_hp_task,
                         const uint32_t* d_lp_task, uint64_t n_scenarios, const fikit_gapfill_params* h_params,
                         const uint64_t* d_gap_offsets, uint64_t n_gaps, uint32_t* d_fill_count, int64_t* d_filled_ns,
                         int64_t* d_lp_completion_ns, uint64_t* d_lp_placed, int32_t* d_status, void* hip_stream) {
  if (!gapfill_params_ok(h_params)) return FIKIT_INVALID_ARG;
  if (!d_task_offsets || !d_task_row_offsets || !d_status || !aligned(d_status, 4)) return FIKIT_INVALID_ARG;
  if (n_scenarios >= MAX_ELEMS || n_gaps >= MAX_ELEMS) return FIKIT_INVALID_ARG;
  if (n_ids > FIKIT_STATIC_MAX_IDS || n_tasks > FIKIT_STATIC_MAX_TASKS) return FIKIT_TOO_LARGE;
  if (n_tasks == 0) return FIKIT_INVALID_ARG;
  if (n_scenarios > 0 && (!d_hp_task || !d_lp_task || !d_gap_offsets || !d_lp_completion_ns || !d_lp_placed))
    return FIKIT_INVALID_ARG;
  if (n_ids > 0 && (!d_ids || !d_rows)) return FIKIT_INVALID_ARG;
  if (n_gaps > 0 && (!d_fill_count || !d_filled_ns)) return FIKIT_INVALID_ARG;
  if (!aligned(d_ids, 8) || !aligned(d_task_offsets, 8) || !aligned(d_rows, 16) || !aligned(d_task_row_offsets, 8) ||
      !aligned(d_hp_task, 4) || !aligned(d_lp_task, 4) || !aligned(d_gap_offsets, 8) || !aligned(d_fill_count, 4) ||
      !aligned(d_filled_ns, 8) || !aligned(d_lp_completion_ns, 8) || !aligned(d_lp_placed, 8))
    return FIKIT_INVALID_ARG;
  unsigned char* ws = nullptr;
  if (int rc = static_scratch_of_current_device(&ws)) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  Tracer tr(st, false);   // (recording events would allocate)
  if (n_scenarios == 0) {
    hipLaunchKernelGGL(k_clear_ctrl, dim3(1), dim3(64), 0, st, reinterpret_cast<Ctrl*>(ws));
  } else if (int rc = gapfill_enqueue(st, tr, d_ids, n_ids, d_task_offsets, n_tasks, d_rows, d_task_row_offsets, d_hp_task,
                                      d_lp_task, n_scenarios, h_params, d_gap_offsets, n_gaps, d_fill_count, d_filled_ns,
                                      d_lp_completion_ns, d_lp_placed, ws, false)) {
    return rc;
  }
  hipLaunchKernelGGL(k_publish_status, dim3(1), dim3(64), 0, st, reinterpret_cast<const Ctrl*>(ws), d_status);
  FIKIT_HIP(hipGetLastError());
  return FIKIT_OK;
}

size_t fikit_measure_workspace_bytes(void) { return 256; }

int fikit_measure(const fikit_launch* d_records, uint64_t n_records, const uint64_t* d_task_offsets, uint32_t n_tasks,
                  int64_t* d_exec_ns, int64_t* d_gap_ns, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  if (!d_task_offsets || !d_workspace) return FIKIT_INVALID_ARG;
  if (n_records >= MAX_ELEMS) return FIKIT_INVALID_ARG;
  if (n_records > 0 && (!d_records || !d_exec_ns || !d_gap_ns || n_tasks == 0)) return FIKIT_INVALID_ARG;
  if (!aligned(d_records, 8) || !aligned(d_task_offsets, 8) || !aligned(d_exec_ns, 8) || !aligned(d_gap_ns, 8) ||
      !aligned(d_workspace, 256))
    return FIKIT_INVALID_ARG;
  if (workspace_bytes < fikit_measure_workspace_bytes()) return FIKIT_WORKSPACE_TOO_SMALL;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  Ctrl* ctrl = static_cast<Ctrl*>(d_workspace);
  Tracer tr(st);
  tr.mark("k_measure");
  hipLaunchKernelGGL(k_clear_ctrl, dim3(1), dim3(64), 0, st, ctrl);
  hipLaunchKernelGGL(k_validate_offsets, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, d_task_offsets, n_tasks, n_records,
                     ctrl);
  if (n_records > 0) {
    hipLaunchKernelGGL(k_measure, dim3(blocks_for(n_records, 256)), dim3(256), 0, st, d_records, n_records, d_exec_ns, d_gap_ns,
                       ctrl);
    hipLaunchKernelGGL(k_measure_task_ends, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, d_task_offsets, n_tasks, d_gap_ns,
                       ctrl);
  }
  FIKIT_HIP(hipGetLastError());
  tr.mark("host_sync");
  Ctrl h{};
  if (int rc = read_ctrl(ctrl, &h, st)) return rc;
  return status_from_bits(h.status);
}

size_t fikit_replay_workspace_bytes(uint64_t n_ids, uint32_t n_tasks, uint64_t n_scenarios) {
  return fikit_gapfill_workspace_bytes(n_ids, n_tasks, n_scenarios);
}

int fikit_gapfill_replay(const uint64_t* d_ids, const uint64_t* d_task_offsets, uint32_t n_tasks, const fikit_row* d_rows,
                         const uint64_t* d_task_row_offsets, const int64_t* d_actual_gap_ns, const uint32_t* d_hp_task,
                         const uint32_t* d_lp_task, uint64_t n_scenarios, const fikit_replay_params* h_params,
                         const uint64_t* d_gap_offsets, uint32_t* d_fill_count, int64_t* d_filled_ns, int64_t* d_hp_delay_ns,
                         uint64_t* d_lp_placed, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  if (!h_params || h_params->margin_ns < 0 || h_params->min_gap_ns < 0 || h_params->predictor < FIKIT_PREDICT_P50 ||
      h_params->predictor > FIKIT_PREDICT_MEAN)
    return FIKIT_INVALID_ARG;
  if (!d_task_offsets || !d_task_row_offsets || !d_workspace) return FIKIT_INVALID_ARG;
  if (n_scenarios >= MAX_ELEMS) return FIKIT_INVALID_ARG;
  if (n_scenarios > 0 && (!d_hp_task || !d_lp_task || !d_gap_offsets || !d_hp_delay_ns || !d_lp_placed || n_tasks == 0))
    return FIKIT_INVALID_ARG;
  if (!aligned(d_ids, 8) || !aligned(d_task_offsets, 8) || !aligned(d_rows, 16) || !aligned(d_task_row_offsets, 8) ||
      !aligned(d_actual_gap_ns, 8) || !aligned(d_hp_task, 4) || !aligned(d_lp_task, 4) || !aligned(d_gap_offsets, 8) ||
      !aligned(d_fill_count, 4) || !aligned(d_filled_ns, 8) || !aligned(d_hp_delay_ns, 8) || !aligned(d_lp_placed, 8) ||
      !aligned(d_workspace, 256))
    return FIKIT_INVALID_ARG;
  if (n_scenarios == 0) return FIKIT_OK;

  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint64_t n_ids = 0, n_gaps = 0;
  FIKIT_HIP(hipMemcpyAsync(&n_ids, d_task_offsets + n_tasks, 8, hipMemcpyDeviceToHost, st));
  FIKIT_HIP(hipMemcpyAsync(&n_gaps, d_gap_offsets + n_scenarios, 8, hipMemcpyDeviceToHost, st));
  FIKIT_HIP(hipStreamSynchronize(st));
  if (n_ids >= MAX_ELEMS || n_gaps >= MAX_ELEMS) return FIKIT_INVALID_ARG;
  if (n_ids > 0 && (!d_ids || !d_rows || !d_actual_gap_ns)) return FIKIT_INVALID_ARG;
  if (n_gaps > 0 && (!d_fill_count || !d_filled_ns)) return FIKIT_INVALID_ARG;
  if (workspace_bytes < fikit_replay_workspace_bytes(n_ids, n_tasks, n_scenarios)) return FIKIT_WORKSPACE_TOO_SMALL;

  unsigned char* ws = static_cast<unsigned char*>(d_workspace);
  Carver c;   // (same layout as fikit_gapfill: the 32-bit arrays share the space of the 64-bit ones)
  Ctrl* ctrl = reinterpret_cast<Ctrl*>(ws + c.take(256));
  uint32_t* role = reinterpret_cast<uint32_t*>(ws + c.take(static_cast<uint64_t>(n_tasks) * 4));
  uint32_t* glists = reinterpret_cast<uint32_t*>(ws + c.take(static_cast<uint64_t>(n_tasks) * 4 * 2));
  uint64_t* lp_total = reinterpret_cast<uint64_t*>(ws + c.take(static_cast<uint64_t>(n_tasks) * 8));
  int64_t* pe = reinterpret_cast<int64_t*>(ws + c.take(n_ids * 8 + GF_PAD));
  int64_t* pg = reinterpret_cast<int64_t*>(ws + c.take(n_ids * 8 + GF_PAD));
  uint32_t* lp_e = reinterpret_cast<uint32_t*>(pe);
  uint2* hp_eg = reinterpret_cast<uint2*>(pg);

  Tracer tr(st);
  tr.mark("gf_setup");
  hipLaunchKernelGGL(k_clear_ctrl, dim3(1), dim3(64), 0, st, ctrl);
  hipLaunchKernelGGL(k_fill_u32, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, role, static_cast<uint64_t>(n_tasks), 0u);
  hipLaunchKernelGGL(k_validate_offsets, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, d_task_offsets, n_tasks, n_ids, ctrl);
  hipLaunchKernelGGL(k_gf_scenarios, dim3(blocks_for(n_scenarios, 256)), dim3(256), 0, st, d_task_offsets, n_tasks, d_hp_task,
                     d_lp_task, n_scenarios, d_gap_offsets, n_gaps, role, ctrl);
  tr.mark("gf_lists");
  hipLaunchKernelGGL(k_gf_lists, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, d_task_offsets, n_tasks, role, 8192u, glists,
                     ctrl);
  tr.mark("k_gf_predict32");
  hipLaunchKernelGGL(k_gf_predict32, dim3(n_tasks), dim3(PRED_THREADS), 0, st, d_ids, d_task_offsets, n_tasks, d_rows,
                     d_task_row_offsets, role, glists, d_actual_gap_ns, lp_e, hp_eg, lp_total,
                     static_cast<uint32_t>(h_params->predictor), static_cast<const uint32_t*>(nullptr), ctrl);
  const uint32_t vec_ok = (aligned(d_fill_count, 16) && aligned(d_filled_ns, 16)) ? 1u : 0u;
  const dim3 grid(blocks_for(n_scenarios, LW_THREADS)), block(LW_THREADS);
  if (h_params->feedback) {
    tr.mark("k_gf_replay_feedback");
    FIKIT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_gf_walk_lanes<LW_REPLAY_FEEDBACK>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(sizeof(LaneWalkSmem))));
    hipLaunchKernelGGL(k_gf_walk_lanes<LW_REPLAY_FEEDBACK>, grid, block, sizeof(LaneWalkSmem), st, d_task_offsets, d_hp_task,
                       d_lp_task, n_scenarios, d_gap_offsets, lp_e, hp_eg, lp_total, h_params->margin_ns, h_params->min_gap_ns,
                       d_fill_count, d_filled_ns, d_hp_delay_ns, d_lp_placed, vec_ok, ctrl);
  } else {
    tr.mark("k_gf_replay");
    FIKIT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_gf_walk_lanes<LW_REPLAY>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(sizeof(LaneWalkSmem))));
    hipLaunchKernelGGL(k_gf_walk_lanes<LW_REPLAY>, grid, block, sizeof(LaneWalkSmem), st, d_task_offsets, d_hp_task, d_lp_task,
                       n_scenarios, d_gap_offsets, lp_e, hp_eg, lp_total, h_params->margin_ns, h_params->min_gap_ns,
                       d_fill_count, d_filled_ns, d_hp_delay_ns, d_lp_placed, vec_ok, ctrl);
  }
  // a prediction that did not fit 32 bits (Ctrl::wide): the walk above has not run; the 64-bit kernels do the call
  tr.mark("k_gf_replay_wide");
  hipLaunchKernelGGL(k_gf_predict, dim3(n_tasks), dim3(PRED_THREADS), 0, st, d_ids, d_task_offsets, n_tasks, d_rows,
                     d_task_row_offsets, role, glists, pe, pg, static_cast<int64_t*>(nullptr), 1u,
                     static_cast<uint32_t>(h_params->predictor), ctrl);
  hipLaunchKernelGGL(k_gf_replay_wide, dim3(blocks_for(n_scenarios, 256)), dim3(256), 0, st, d_task_offsets, d_hp_task, d_lp_task,
                     n_scenarios, d_gap_offsets, pe, pg, d_actual_gap_ns, h_params->margin_ns, h_params->min_gap_ns,
                     h_params->feedback ? 1u : 0u, d_fill_count, d_filled_ns, d_hp_delay_ns, d_lp_placed, ctrl);
  FIKIT_HIP(hipGetLastError());
  tr.mark("host_sync");
  Ctrl h{};
  if (int rc = read_ctrl(ctrl, &h, st)) return rc;
  return status_from_bits(h.status);
}

size_t fikit_prio_fill_workspace_bytes(uint64_t n_ids, uint32_t n_tasks, uint64_t n_scenarios) {
  (void)n_scenarios;
  if (n_ids >= MAX_ELEMS) return 0;
  Carver c;
  c.take(256);
  c.take(static_cast<uint64_t>(n_tasks) * 4);
  c.take(static_cast<uint64_t>(n_tasks) * 4 * 2);
  c.take(static_cast<uint64_t>(n_tasks) * 8);
  c.take(n_ids * 8 + GF_PAD);
  c.take(n_ids * 8 + GF_PAD);
  return static_cast<size_t>(c.at);
}

int fikit_prio_fill(const uint64_t* d_ids, const uint64_t* d_task_offsets, uint32_t n_tasks, const fikit_row* d_rows,
                    const uint64_t* d_task_row_offsets, const uint32_t* d_hp_task, const uint64_t* d_lp_offsets,
                    const uint32_t* d_lp_task, const uint32_t* d_lp_prio, uint64_t n_scenarios,
                    const fikit_gapfill_params* h_params, const uint64_t* d_gap_offsets, uint32_t* d_fill_count,
                    int64_t* d_filled_ns, uint64_t* d_lp_placed, int64_t* d_lp_placed_ns, void* d_workspace,
                    size_t workspace_bytes, void* hip_stream) {
  if (!h_params || h_params->margin_ns < 0 || h_params->min_gap_ns < 0 || h_params->reserved != 0 ||
      h_params->predictor < FIKIT_PREDICT_P50 || h_params->predictor > FIKIT_PREDICT_MEAN)
    return FIKIT_INVALID_ARG;
  if (!d_task_offsets || !d_task_row_offsets || !d_workspace) return FIKIT_INVALID_ARG;
  if (n_scenarios >= MAX_ELEMS / FIKIT_PRIO_MAX_LP) return FIKIT_INVALID_ARG;
  if (n_scenarios > 0 && (!d_hp_task || !d_lp_offsets || !d_gap_offsets || n_tasks == 0)) return FIKIT_INVALID_ARG;
  if (!aligned(d_ids, 8) || !aligned(d_task_offsets, 8) || !aligned(d_rows, 16) || !aligned(d_task_row_offsets, 8) ||
      !aligned(d_hp_task, 4) || !aligned(d_lp_offsets, 8) || !aligned(d_lp_task, 4) || !aligned(d_lp_prio, 4) ||
      !aligned(d_gap_offsets, 8) || !aligned(d_fill_count, 4) || !aligned(d_filled_ns, 8) || !aligned(d_lp_placed, 8) ||
      !aligned(d_lp_placed_ns, 8) || !aligned(d_workspace, 256))
    return FIKIT_INVALID_ARG;
  if (n_scenarios == 0) return FIKIT_OK;

  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint64_t n_ids = 0, n_gaps = 0, n_entries = 0;
  FIKIT_HIP(hipMemcpyAsync(&n_ids, d_task_offsets + n_tasks, 8, hipMemcpyDeviceToHost, st));
  FIKIT_HIP(hipMemcpyAsync(&n_gaps, d_gap_offsets + n_scenarios, 8, hipMemcpyDeviceToHost, st));
  FIKIT_HIP(hipMemcpyAsync(&n_entries, d_lp_offsets + n_scenarios, 8, hipMemcpyDeviceToHost, st));
  FIKIT_HIP(hipStreamSynchronize(st));
  if (n_ids >= MAX_ELEMS || n_gaps >= MAX_ELEMS || n_entries >= MAX_ELEMS) return FIKIT_INVALID_ARG;
  if (n_ids > 0 && (!d_ids || !d_rows)) return FIKIT_INVALID_ARG;
  if (n_gaps > 0 && (!d_fill_count || !d_filled_ns)) return FIKIT_INVALID_ARG;
  if (n_entries > 0 && (!d_lp_task || !d_lp_prio || !d_lp_placed || !d_lp_placed_ns)) return FIKIT_INVALID_ARG;
  if (workspace_bytes < fikit_prio_fill_workspace_bytes(n_ids, n_tasks, n_scenarios)) return FIKIT_WORKSPACE_TOO_SMALL;

  unsigned char* ws = static_cast<unsigned char*>(d_workspace);
  Carver c;
  Ctrl* ctrl = reinterpret_cast<Ctrl*>(ws + c.take(256));
  uint32_t* role = reinterpret_cast<uint32_t*>(ws + c.take(static_cast<uint64_t>(n_tasks) * 4));
  uint32_t* glists = reinterpret_cast<uint32_t*>(ws + c.take(static_cast<uint64_t>(n_tasks) * 4 * 2));
  uint64_t* lp_total = reinterpret_cast<uint64_t*>(ws + c.take(static_cast<uint64_t>(n_tasks) * 8));
  int64_t* pe = reinterpret_cast<int64_t*>(ws + c.take(n_ids * 8 + GF_PAD));   // the 32-bit arrays share the space of the 64-bit ones
  int64_t* pg = reinterpret_cast<int64_t*>(ws + c.take(n_ids * 8 + GF_PAD));
  uint32_t* lp_e = reinterpret_cast<uint32_t*>(pe);
  uint2* hp_eg = reinterpret_cast<uint2*>(pg);

  Tracer tr(st);
  tr.mark("pf_setup");
  hipLaunchKernelGGL(k_clear_ctrl, dim3(1), dim3(64), 0, st, ctrl);
  hipLaunchKernelGGL(k_fill_u32, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, role, static_cast<uint64_t>(n_tasks), 0u);
  hipLaunchKernelGGL(k_validate_offsets, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, d_task_offsets, n_tasks, n_ids, ctrl);
  hipLaunchKernelGGL(k_pf_scenarios, dim3(blocks_for(n_scenarios, 256)), dim3(256), 0, st, d_task_offsets, n_tasks, d_hp_task,
                     d_lp_offsets, d_lp_task, d_lp_prio, n_scenarios, n_entries, d_gap_offsets, role, ctrl);
  hipLaunchKernelGGL(k_gf_lists, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, d_task_offsets, n_tasks, role, 8192u, glists,
                     ctrl);
  FIKIT_HIP(hipGetLastError());
  tr.mark("host_sync");
  Ctrl h{};
  if (int rc = read_ctrl(ctrl, &h, st)) return rc;   // the widest scenario decides how many lanes share one
  if (int rc = status_from_bits(h.status)) return rc;
  const uint32_t widest = h.n_class[3];
  // Up to 64 low-priority tasks per scenario: a group of lanes per scenario on 32-bit predictions; the 64-bit
  // kernels then only run if a prediction did not fit (they check Ctrl::wide).  More tasks: the 64-bit kernels.
  const bool groups = widest <= PF_MAX_LP;
  if (groups) {
    tr.mark("k_gf_predict32");
    hipLaunchKernelGGL(k_gf_predict32, dim3(n_tasks), dim3(PRED_THREADS), 0, st, d_ids, d_task_offsets, n_tasks, d_rows,
                       d_task_row_offsets, role, glists, static_cast<const int64_t*>(nullptr), lp_e, hp_eg, lp_total,
                       static_cast<uint32_t>(h_params->predictor), static_cast<const uint32_t*>(nullptr), ctrl);
    const uint32_t vec_ok = (aligned(d_fill_count, 16) && aligned(d_filled_ns, 16)) ? 1u : 0u;
    tr.mark("k_pf_walk");
    int rc = FIKIT_OK;
#define FIKIT_PF_WALK(W)                                                                                                   \
  rc = launch_prio_walk<W>(st, d_task_offsets, d_hp_task, d_lp_offsets, d_lp_task, d_lp_prio, n_scenarios, d_gap_offsets, \
                           lp_e, hp_eg, h_params->margin_ns, h_params->min_gap_ns, d_fill_count, d_filled_ns, d_lp_placed, \
                           d_lp_placed_ns, vec_ok, ctrl)
    if (widest <= 1) FIKIT_PF_WALK(1);
    else if (widest <= 2) FIKIT_PF_WALK(2);
    else if (widest <= 4) FIKIT_PF_WALK(4);
    else if (widest <= 8) FIKIT_PF_WALK(8);
    else if (widest <= 16) FIKIT_PF_WALK(16);
    else if (widest <= 32) FIKIT_PF_WALK(32);
    else FIKIT_PF_WALK(64);
#undef FIKIT_PF_WALK
    if (rc) return rc;
  }
  const uint32_t only_if_wide = groups ? 1u : 0u;
  tr.mark("k_pf_walk_wide");
  hipLaunchKernelGGL(k_gf_predict, dim3(n_tasks), dim3(PRED_THREADS), 0, st, d_ids, d_task_offsets, n_tasks, d_rows,
                     d_task_row_offsets, role, glists, pe, pg, static_cast<int64_t*>(nullptr), only_if_wide,
                     static_cast<uint32_t>(h_params->predictor), ctrl);
  hipLaunchKernelGGL(k_pf_walk_wide, dim3(blocks_for(n_scenarios, 64)), dim3(64), 0, st, d_task_offsets, d_hp_task, d_lp_offsets,
                     d_lp_task, d_lp_prio, n_scenarios, d_gap_offsets, pe, pg, h_params->margin_ns, h_params->min_gap_ns,
                     d_fill_count, d_filled_ns, d_lp_placed, d_lp_placed_ns, only_if_wide, ctrl);
  FIKIT_HIP(hipGetLastError());
  tr.mark("host_sync");
  if (int rc2 = read_ctrl(ctrl, &h, st)) return rc2;
  return status_from_bits(h.status);
}

size_t fikit_pairing_workspace_bytes(uint32_t n_tasks) {
  Carver c;
  c.take(256);
  c.take(static_cast<uint64_t>(n_tasks) * 8);
  return static_cast<size_t>(c.at);
}

int fikit_pairing_best(const uint32_t* d_hp_task, const uint32_t* d_lp_task, uint64_t n_scenarios, uint32_t n_tasks,
                       const uint64_t* d_gap_offsets, const int64_t* d_filled_ns, const int64_t* d_lp_completion_ns,
                       int64_t* d_scenario_filled_ns, uint64_t* d_best_scenario, uint32_t* d_best_lp,
                       int64_t* d_best_filled_ns, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  if (!d_workspace || n_scenarios >= (1ull << 31)) return FIKIT_INVALID_ARG;   // (one workgroup per scenario)
  if (n_tasks > 0 && (!d_best_scenario || !d_best_lp || !d_best_filled_ns)) return FIKIT_INVALID_ARG;
  if (n_scenarios > 0 &&
      (!d_hp_task || !d_lp_task || !d_gap_offsets || !d_lp_completion_ns || !d_scenario_filled_ns || n_tasks == 0))
    return FIKIT_INVALID_ARG;
  if (!aligned(d_hp_task, 4) || !aligned(d_lp_task, 4) || !aligned(d_gap_offsets, 8) || !aligned(d_filled_ns, 8) ||
      !aligned(d_lp_completion_ns, 8) || !aligned(d_scenario_filled_ns, 8) || !aligned(d_best_scenario, 8) ||
      !aligned(d_best_lp, 4) || !aligned(d_best_filled_ns, 8) || !aligned(d_workspace, 256))
    return FIKIT_INVALID_ARG;
  if (workspace_bytes < fikit_pairing_workspace_bytes(n_tasks)) return FIKIT_WORKSPACE_TOO_SMALL;
  if (n_tasks == 0) return FIKIT_OK;

  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint64_t n_gaps = 0;
  if (n_scenarios > 0) {
    FIKIT_HIP(hipMemcpyAsync(&n_gaps, d_gap_offsets + n_scenarios, 8, hipMemcpyDeviceToHost, st));
    FIKIT_HIP(hipStreamSynchronize(st));
    if (n_gaps >= MAX_ELEMS || (n_gaps > 0 && !d_filled_ns)) return FIKIT_INVALID_ARG;
  }
  unsigned char* ws = static_cast<unsigned char*>(d_workspace);
  Carver c;
  Ctrl* ctrl = reinterpret_cast<Ctrl*>(ws + c.take(256));
  long long* soonest = reinterpret_cast<long long*>(ws + c.take(static_cast<uint64_t>(n_tasks) * 8));
  long long* top_filled = reinterpret_cast<long long*>(d_best_filled_ns);
  unsigned long long* best_scenario = reinterpret_cast<unsigned long long*>(d_best_scenario);

  Tracer tr(st);
  tr.mark("pair_setup");
  hipLaunchKernelGGL(k_clear_ctrl, dim3(1), dim3(64), 0, st, ctrl);
  hipLaunchKernelGGL(k_pair_init, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, n_tasks, top_filled, soonest, best_scenario);
  if (n_scenarios > 0) {
    tr.mark("k_pair_sum");
    hipLaunchKernelGGL(k_pair_sum, dim3(static_cast<uint32_t>(n_scenarios)), dim3(PAIR_THREADS), 0, st, d_hp_task, d_lp_task,
                       n_scenarios, n_tasks, d_gap_offsets, n_gaps, d_filled_ns, d_scenario_filled_ns, top_filled, ctrl);
    tr.mark("k_pair_pick");
    hipLaunchKernelGGL(k_pair_soonest, dim3(blocks_for(n_scenarios, 256)), dim3(256), 0, st, d_hp_task, n_scenarios,
                       d_scenario_filled_ns, d_lp_completion_ns, top_filled, soonest, ctrl);
    hipLaunchKernelGGL(k_pair_first, dim3(blocks_for(n_scenarios, 256)), dim3(256), 0, st, d_hp_task, n_scenarios,
                       d_scenario_filled_ns, d_lp_completion_ns, top_filled, soonest, best_scenario, ctrl);
  }
  hipLaunchKernelGGL(k_pair_finish, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, n_tasks, d_lp_task, best_scenario,
                     d_best_lp, top_filled, ctrl);
  FIKIT_HIP(hipGetLastError());
  tr.mark("host_sync");
  Ctrl h{};
  if (int rc = read_ctrl(ctrl, &h, st)) return rc;
  return status_from_bits(h.status);
}

size_t fikit_profile_merge_workspace_bytes(uint32_t n_tasks) {
  Carver c;
  c.take(256);
  c.take((static_cast<uint64_t>(n_tasks) + 1) * 4);
  c.take(((static_cast<uint64_t>(n_tasks) + 1) / SCAN_TILE + 2) * 4);
  return static_cast<size_t>(c.at);
}

int fikit_profile_merge(const fikit_row* d_rows_a, const uint64_t* d_task_row_offsets_a, const fikit_row* d_rows_b,
                        const uint64_t* d_task_row_offsets_b, uint32_t n_tasks, fikit_row* d_rows_out, uint64_t row_capacity,
                        uint64_t* d_task_row_offsets_out, uint64_t* h_n_rows, void* d_workspace, size_t workspace_bytes,
                        void* hip_stream) {
  if (h_n_rows) *h_n_rows = 0;
  if (!h_n_rows || !d_task_row_offsets_a || !d_task_row_offsets_b || !d_task_row_offsets_out || !d_workspace || n_tasks == 0)
    return FIKIT_INVALID_ARG;
  if (row_capacity > 0 && !d_rows_out) return FIKIT_INVALID_ARG;
  if (!aligned(d_rows_a, 16) || !aligned(d_rows_b, 16) || !aligned(d_rows_out, 16) || !aligned(d_task_row_offsets_a, 8) ||
      !aligned(d_task_row_offsets_b, 8) || !aligned(d_task_row_offsets_out, 8) || !aligned(d_workspace, 256))
    return FIKIT_INVALID_ARG;
  if (workspace_bytes < fikit_profile_merge_workspace_bytes(n_tasks)) return FIKIT_WORKSPACE_TOO_SMALL;

  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint64_t na = 0, nb = 0;
  FIKIT_HIP(hipMemcpyAsync(&na, d_task_row_offsets_a + n_tasks, 8, hipMemcpyDeviceToHost, st));
  FIKIT_HIP(hipMemcpyAsync(&nb, d_task_row_offsets_b + n_tasks, 8, hipMemcpyDeviceToHost, st));
  FIKIT_HIP(hipStreamSynchronize(st));
  if (na >= MAX_ELEMS || nb >= MAX_ELEMS || na + nb >= MAX_ELEMS) return FIKIT_INVALID_ARG;
  if ((na > 0 && !d_rows_a) || (nb > 0 && !d_rows_b)) return FIKIT_INVALID_ARG;

  unsigned char* ws = static_cast<unsigned char*>(d_workspace);
  Carver c;
  Ctrl* ctrl = reinterpret_cast<Ctrl*>(ws + c.take(256));
  uint32_t* dcount = reinterpret_cast<uint32_t*>(ws + c.take((static_cast<uint64_t>(n_tasks) + 1) * 4));
  uint32_t* sums = reinterpret_cast<uint32_t*>(ws + c.take(((static_cast<uint64_t>(n_tasks) + 1) / SCAN_TILE + 2) * 4));

  Tracer tr(st);
  tr.mark("merge_count");
  const uint32_t grid = n_tasks < 65536u ? n_tasks : 65536u;
  hipLaunchKernelGGL(k_clear_ctrl, dim3(1), dim3(64), 0, st, ctrl);
  hipLaunchKernelGGL(k_validate_offsets, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, d_task_row_offsets_a, n_tasks, na, ctrl);
  hipLaunchKernelGGL(k_validate_offsets, dim3(blocks_for(n_tasks, 256)), dim3(256), 0, st, d_task_row_offsets_b, n_tasks, nb, ctrl);
  hipLaunchKernelGGL(k_merge<0>, dim3(grid), dim3(MERGE_THREADS), 0, st, d_rows_a, d_task_row_offsets_a, d_rows_b,
                     d_task_row_offsets_b, n_tasks, dcount, static_cast<const uint64_t*>(nullptr),
                     static_cast<fikit_row*>(nullptr), ctrl);
  if (int rc = scan_u32(dcount, static_cast<uint64_t>(n_tasks) + 1, sums, &ctrl->n_rows, st)) return rc;
  hipLaunchKernelGGL(k_widen_offsets, dim3(blocks_for(static_cast<uint64_t>(n_tasks) + 1, 256)), dim3(256), 0, st, dcount,
                     static_cast<uint64_t>(n_tasks) + 1, d_task_row_offsets_out);
  FIKIT_HIP(hipGetLastError());
  tr.mark("host_sync");
  Ctrl h{};
  if (int rc = read_ctrl(ctrl, &h, st)) return rc;
  if (int rc = status_from_bits(h.status)) return rc;
  *h_n_rows = h.n_rows;
  if (h.n_rows > row_capacity) return FIKIT_ROW_CAPACITY;
  tr.mark("k_merge_rows");
  hipLaunchKernelGGL(k_merge<1>, dim3(grid), dim3(MERGE_THREADS), 0, st, d_rows_a, d_task_row_offsets_a, d_rows_b,
                     d_task_row_offsets_b, n_tasks, dcount, d_task_row_offsets_out, d_rows_out, ctrl);
  FIKIT_HIP(hipGetLastError());
  FIKIT_HIP(hipStreamSynchronize(st));
  return FIKIT_OK;
}

}  // extern "C"
