// CPU oracle for the FIKIT trace-profiling and gap-filling path.
//
// TEST INFRASTRUCTURE ONLY.  This file is the definition of "correct" that the GPU library is
// compared against.  It is plain, single-threaded and slow on purpose, and it shares nothing
// with the GPU library: no header, no helper, no table.  Only tests, the smoke check and the
// benchmark's CPU-baseline leg may call it; the product never does.
//
// What it computes, and where the paper defines it (arXiv 2311.10359):
//
//   oracle_kernel_id  - the Kernel ID of a launch (Section 3.2, "Identifying each kernel": the
//                       kernel's function name, block dimensions and grid dimensions make up its
//                       ID).  The ID here is the 64-bit FNV-1a hash of the 32 bytes that hold
//                       name id, grid[3], block[3] and dynamic shared-memory bytes.
//   oracle_profile    - the measurement phase's statistical output (Section 3.2, "Data
//                       acquisition and statistical output during the measurement phase"): the
//                       set of unique IDs S_UID of each task, and per ID the execution times
//                       K and the idle times G that follow a kernel of that ID, over all measured
//                       runs of the task (a launch record names its run; a run of N kernels has
//                       N - 1 idle times, none between one run and the next).  The paper
//                       prints the means SK_j and SG_j; this oracle emits count and sum (so the
//                       mean is sum/count) and, beyond the paper, min, max and nearest-rank p50
//                       and p95 of the same samples.
//   oracle_gapfill    - Algorithm 1 (FIKIT procedure) with Algorithm 2 (BestPrioFit) in the
//                       case of one high-priority and one low-priority task: the low-priority
//                       task's waiting queue then holds exactly one request at a time, its next
//                       kernel, so "best fit" degenerates to first-in-first-out and a gap ends
//                       as soon as that head request does not fit.
//   oracle_measure    - the two per-launch measurements of Section 3.2 ("Measuring the execution
//                       and idle time of kernel"): execution time K and the idle time G that
//                       follows a launch, as they stand in the trace.
//   oracle_replay     - the same filling procedure played against the idle times that actually
//                       occurred ("Real time feedback to stop error propagation", end of the
//                       scheduling section, Figure "Runtime Feedback"): without feedback every
//                       kernel that fits the predicted gap is issued and what runs past the
//                       actual gap delays the high-priority task (overhead 1); with feedback the
//                       controller stops issuing once the next high-priority request has
//                       arrived, and only the kernel already issued can run over (overhead 2).
//   oracle_prio_fill  - Algorithm 1 with the full Algorithm 2 (BestPrioFit): several low-priority
//                       tasks wait in the priority queues Q1..Q9, each with one request at a time
//                       (its next kernel); per gap the procedure keeps taking, from the highest
//                       priority level that has a request that fits, the request that fits best
//                       (the longest), until nothing fits.
//   oracle_pairing_best - the question of the paper's discussion section ("What Tasks are Suitable
//                       for Sharing a GPU": measure combinations of tasks beforehand, then find for
//                       a task its best matching partner in those measurements): over evaluated
//                       (high-priority, low-priority) combinations, per high-priority task the
//                       partner whose kernels fill the most of its idle time.
//   oracle_profile_merge - the statistics of the measurement phase accumulated over runs (Section 3.2: the
//                       sums of SK_j and SG_j run over the T measured runs of a task, and a run of N
//                       kernels contributes N - 1 idle times): the profile of further runs is merged
//                       into the profile of the runs so far.
//
// All quantities are integers (nanoseconds, counts); nothing is floating point.

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <map>
#include <vector>

namespace {

// Input record, 64 bytes, little endian (own definition; mirrors the documented layout).
struct Launch {
  uint32_t name_id;
  uint32_t grid[3];
  uint32_t block[3];
  uint32_t shmem;
  int64_t start_ns;
  int64_t end_ns;
  uint32_t run;  // which of the task's measured runs the launch belongs to (not part of the identity)
  uint8_t reserved[12];
};
static_assert(sizeof(Launch) == 64, "launch record is 64 bytes");

struct Stats {
  uint64_t count;
  uint64_t sum;
  int64_t min, max, p50, p95;
};
static_assert(sizeof(Stats) == 48, "stats block is 48 bytes");

struct Row {
  uint64_t kernel_id;
  uint32_t task;
  uint32_t reserved0;
  Stats exec;
  Stats gap;
  uint8_t reserved1[16];
};
static_assert(sizeof(Row) == 128, "row is 128 bytes");

enum : int {
  OK = 0,
  INVALID_ARG = -1,
  ROW_CAPACITY = -3,
  BAD_RECORD = -4,
  UNKNOWN_ID = -5,
};

// FNV-1a, 64 bit: start from the offset basis; for every byte, xor it in, then multiply by
// the FNV prime, modulo 2^64.
uint64_t fnv1a64(const uint8_t* p, size_t len) {
  uint64_t h = 0xcbf29ce484222325ull;
  for (size_t i = 0; i < len; ++i) {
    h ^= static_cast<uint64_t>(p[i]);
    h *= 0x100000001b3ull;
  }
  return h;
}

// Nearest-rank percentile of an ascending vector: the value at 1-based rank ceil(K*n/100).
int64_t nearest_rank(const std::vector<int64_t>& sorted, uint64_t k) {
  uint64_t n = sorted.size();
  uint64_t rank = (k * n + 99) / 100;  // ceil(k*n/100)
  return sorted[rank - 1];
}

Stats stats_of(std::vector<int64_t> v) {
  Stats s;
  std::memset(&s, 0, sizeof(s));
  if (v.empty()) return s;  // an ID seen only as a task's last launch has no idle-time sample
  std::sort(v.begin(), v.end());
  s.count = v.size();
  uint64_t sum = 0;
  for (int64_t x : v) sum += static_cast<uint64_t>(x);  // modulo 2^64
  s.sum = sum;
  s.min = v.front();
  s.max = v.back();
  s.p50 = nearest_rank(v, 50);
  s.p95 = nearest_rank(v, 95);
  return s;
}

// The predicted duration taken from a row's statistics: the nearest-rank median (predictor 0), or the
// mean the paper defines, SK_j / SG_j of Section 3.2 = sum / count, rounded down to whole nanoseconds
// (predictor 1; 0 if there is no sample).
int64_t predicted(const Stats& s, int predictor) {
  if (predictor == 0) return s.p50;
  return s.count ? static_cast<int64_t>(s.sum / s.count) : 0;
}

struct Samples {
  std::vector<int64_t> exec;  // K: execution time of every launch with this ID
  std::vector<int64_t> gap;   // G: idle time after every launch with this ID (not the last of a run)
};

bool offsets_ok(const uint64_t* off, uint32_t n_tasks, uint64_t n) {
  if (!off) return false;
  if (off[0] != 0) return false;
  for (uint32_t t = 0; t < n_tasks; ++t)
    if (off[t + 1] < off[t]) return false;
  return off[n_tasks] == n;
}

}  // namespace

extern "C" {

uint64_t oracle_kernel_id(const uint8_t* bytes, uint64_t len) { return fnv1a64(bytes, len); }

// Measurement-phase statistics.  rows_out receives one Row per (task, unique ID), tasks
// ascending, IDs ascending as unsigned numbers; task_row_offsets[t]..[t+1] delimit task t's rows.
// ids_out (may be null) receives every launch's ID in launch order.
int oracle_profile(const void* records_v, uint64_t n_records, const uint64_t* task_offsets,
                   uint32_t n_tasks, uint64_t* ids_out, void* rows_out_v, uint64_t row_capacity,
                   uint64_t* task_row_offsets, uint64_t* n_rows_out) {
  const Launch* rec = static_cast<const Launch*>(records_v);
  Row* rows = static_cast<Row*>(rows_out_v);
  if (!n_rows_out || !task_row_offsets) return INVALID_ARG;
  if (n_records && !rec) return INVALID_ARG;
  if (!offsets_ok(task_offsets, n_tasks, n_records)) return INVALID_ARG;

  uint64_t n_rows = 0;
  bool overflow = false;
  for (uint32_t t = 0; t < n_tasks; ++t) {
    task_row_offsets[t] = n_rows;
    std::map<uint64_t, Samples> by_id;  // S_UID of this task, ordered by unsigned ID
    const uint64_t lo = task_offsets[t], hi = task_offsets[t + 1];
    for (uint64_t i = lo; i < hi; ++i) {
      const uint64_t id = fnv1a64(reinterpret_cast<const uint8_t*>(&rec[i]), 32);
      if (ids_out) ids_out[i] = id;
      if (rec[i].end_ns < rec[i].start_ns) return BAD_RECORD;
      const int64_t k = rec[i].end_ns - rec[i].start_ns;  // execution time K
      Samples& s = by_id[id];
      s.exec.push_back(k);
      // idle time G: from this kernel's end to the next kernel's start; a run of N kernels has N - 1 of them
      // (Section 3.2), so the last kernel of a run has none even if another run of the task follows
      if (i + 1 < hi && rec[i + 1].run == rec[i].run) {
        int64_t g = rec[i + 1].start_ns - rec[i].end_ns;
        if (g < 0) g = 0;  // overlapping kernels leave no idle time
        s.gap.push_back(g);
      }
    }
    for (auto& kv : by_id) {
      if (n_rows < row_capacity && rows) {
        Row r;
        std::memset(&r, 0, sizeof(r));
        r.kernel_id = kv.first;
        r.task = t;
        r.exec = stats_of(kv.second.exec);
        r.gap = stats_of(kv.second.gap);
        rows[n_rows] = r;
      } else {
        overflow = true;
      }
      ++n_rows;
    }
  }
  task_row_offsets[n_tasks] = n_rows;
  *n_rows_out = n_rows;
  return overflow ? ROW_CAPACITY : OK;
}

// Gap filling, one (high-priority task, low-priority task) pair per scenario.
//
// Predictions come from the profile rows: a launch's predicted execution time is the p50
// execution time of its ID, the predicted idle time after a high-priority launch is the p50
// idle time of its ID (predictor 0), or the means SK_j and SG_j of Section 3.2 (predictor 1).  Per high-priority gap the procedure (Algorithm 1) skips gaps below
// min_gap_ns, reserves margin_ns at the end of the gap, and then keeps issuing the
// low-priority task's next kernel while its predicted duration does not exceed what is left,
// subtracting each issued kernel's duration from the remaining idle time.
//
// Outputs per gap: number of low-priority kernels issued and nanoseconds filled.  Per scenario:
// how many low-priority kernels went into gaps, and the time (on the predicted timeline that
// starts at 0 with the first high-priority kernel) at which the low-priority task finishes;
// kernels that found no gap run back to back after the last high-priority kernel.
// assign (optional, indexed through assign_offsets[S+1]) receives for every low-priority launch
// the gap it was put in, or 0xffffffff if it ran after the high-priority trace.
int oracle_gapfill(const uint64_t* ids, const uint64_t* task_offsets, uint32_t n_tasks,
                   const void* rows_v, const uint64_t* task_row_offsets, const uint32_t* hp_task,
                   const uint32_t* lp_task, uint64_t n_scenarios, int64_t margin_ns,
                   int64_t min_gap_ns, const uint64_t* gap_offsets, uint32_t* fill_count,
                   int64_t* filled_ns, int64_t* lp_completion_ns, uint64_t* lp_placed,
                   const uint64_t* assign_offsets, uint32_t* assign, int predictor) {
  const Row* rows = static_cast<const Row*>(rows_v);
  if (!task_offsets || !task_row_offsets) return INVALID_ARG;
  if (n_scenarios && (!hp_task || !lp_task || !gap_offsets || !lp_completion_ns || !lp_placed))
    return INVALID_ARG;
  if (margin_ns < 0 || min_gap_ns < 0 || predictor < 0 || predictor > 1) return INVALID_ARG;

  for (uint64_t s = 0; s < n_scenarios; ++s) {
    const uint32_t hp = hp_task[s], lp = lp_task[s];
    if (hp >= n_tasks || lp >= n_tasks) return INVALID_ARG;

    // Load the profiled data of the two tasks, keyed by Kernel ID.
    std::map<uint64_t, const Row*> hp_rows, lp_rows;
    for (uint64_t r = task_row_offsets[hp]; r < task_row_offsets[hp + 1]; ++r)
      hp_rows[rows[r].kernel_id] = &rows[r];
    for (uint64_t r = task_row_offsets[lp]; r < task_row_offsets[lp + 1]; ++r)
      lp_rows[rows[r].kernel_id] = &rows[r];

    const uint64_t h0 = task_offsets[hp], H = task_offsets[hp + 1] - h0;
    const uint64_t l0 = task_offsets[lp], L = task_offsets[lp + 1] - l0;

    std::vector<int64_t> D(L);  // predicted duration of each low-priority kernel
    for (uint64_t j = 0; j < L; ++j) {
      auto it = lp_rows.find(ids[l0 + j]);
      if (it == lp_rows.end()) return UNKNOWN_ID;
      D[j] = predicted(it->second->exec, predictor);
    }

    uint64_t p = 0;        // next low-priority kernel to issue (FIFO)
    int64_t t = 0;         // predicted time
    bool done = (L == 0);  // low-priority task finished
    int64_t completion = 0;
    const uint64_t g0 = gap_offsets[s];
    for (uint64_t i = 0; i < H; ++i) {
      auto it = hp_rows.find(ids[h0 + i]);
      if (it == hp_rows.end()) return UNKNOWN_ID;
      const int64_t E = predicted(it->second->exec, predictor);
      const int64_t G = predicted(it->second->gap, predictor);
      t += E;  // high-priority kernel i runs and ends at t
      if (i + 1 == H) break;  // no gap after the last launch
      uint32_t c = 0;
      int64_t f = 0;
      if (G >= min_gap_ns && G >= margin_ns) {
        int64_t r = G - margin_ns;  // remaining idle time
        while (p < L && D[p] <= r) {
          r -= D[p];
          f += D[p];
          if (assign) assign[assign_offsets[s] + p] = static_cast<uint32_t>(i);
          ++p;
          ++c;
        }
        if (p == L && c > 0 && !done) {
          completion = t + f;
          done = true;
        }
      }
      fill_count[g0 + i] = c;
      filled_ns[g0 + i] = f;
      t += G;  // the high-priority timeline is never delayed
    }
    lp_placed[s] = p;
    if (!done) {
      int64_t rest = 0;
      for (uint64_t j = p; j < L; ++j) {
        rest += D[j];
        if (assign) assign[assign_offsets[s] + j] = 0xffffffffu;
      }
      completion = t + rest;
    }
    lp_completion_ns[s] = completion;
  }
  return OK;
}

// Execution time K = end - start of every launch, and the idle time G = max(0, next start - end)
// that follows it inside its task; the last launch of a task has no idle time: -1.
int oracle_measure(const void* records_v, uint64_t n_records, const uint64_t* task_offsets,
                   uint32_t n_tasks, int64_t* exec_ns, int64_t* gap_ns) {
  const Launch* rec = static_cast<const Launch*>(records_v);
  if (n_records && (!rec || !exec_ns || !gap_ns)) return INVALID_ARG;
  if (!offsets_ok(task_offsets, n_tasks, n_records)) return INVALID_ARG;
  for (uint32_t t = 0; t < n_tasks; ++t) {
    const uint64_t lo = task_offsets[t], hi = task_offsets[t + 1];
    for (uint64_t i = lo; i < hi; ++i) {
      if (rec[i].end_ns < rec[i].start_ns) return BAD_RECORD;
      exec_ns[i] = rec[i].end_ns - rec[i].start_ns;
      int64_t g = -1;
      if (i + 1 < hi && rec[i + 1].run == rec[i].run) {  // (no idle time after the last kernel of a run)
        g = rec[i + 1].start_ns - rec[i].end_ns;
        if (g < 0) g = 0;
      }
      gap_ns[i] = g;
    }
  }
  return OK;
}

// Gap filling replayed against the actual idle times of the high-priority trace.
//
// Decisions are taken as in oracle_gapfill, on predictions: a gap whose predicted length is below
// min_gap_ns or margin_ns is skipped, and a low-priority kernel is issued only while its predicted
// duration fits what is left of the predicted gap minus the margin.  Issued kernels run back to
// back from the start of the gap and take their predicted duration.  actual_gap_ns[i] is the idle
// time that really followed high-priority launch i (as oracle_measure gives it).
//   feedback == 0: every kernel that fits the prediction is issued.
//   feedback != 0: before each issue the controller looks whether the next high-priority request
//                  has arrived, i.e. whether the time already filled in this gap has reached the
//                  actual idle time; if so it stops issuing for this gap.
// In both cases the time by which the issued kernels run past the actual idle time delays the next
// high-priority kernel; hp_delay_ns[s] is the sum of these delays over the scenario's gaps (the
// paper's overhead 1 without feedback, overhead 2 with it).  Each gap is charged on its own: the
// replay does not shift later launches of the trace.
int oracle_replay(const uint64_t* ids, const uint64_t* task_offsets, uint32_t n_tasks,
                  const void* rows_v, const uint64_t* task_row_offsets, const int64_t* actual_gap_ns,
                  const uint32_t* hp_task, const uint32_t* lp_task, uint64_t n_scenarios,
                  int64_t margin_ns, int64_t min_gap_ns, int feedback, const uint64_t* gap_offsets,
                  uint32_t* fill_count, int64_t* filled_ns, int64_t* hp_delay_ns, uint64_t* lp_placed,
                  int predictor) {
  const Row* rows = static_cast<const Row*>(rows_v);
  if (!task_offsets || !task_row_offsets) return INVALID_ARG;
  if (n_scenarios && (!hp_task || !lp_task || !gap_offsets || !hp_delay_ns || !lp_placed)) return INVALID_ARG;
  if (margin_ns < 0 || min_gap_ns < 0 || predictor < 0 || predictor > 1) return INVALID_ARG;

  for (uint64_t s = 0; s < n_scenarios; ++s) {
    const uint32_t hp = hp_task[s], lp = lp_task[s];
    if (hp >= n_tasks || lp >= n_tasks) return INVALID_ARG;
    std::map<uint64_t, const Row*> hp_rows, lp_rows;
    for (uint64_t r = task_row_offsets[hp]; r < task_row_offsets[hp + 1]; ++r) hp_rows[rows[r].kernel_id] = &rows[r];
    for (uint64_t r = task_row_offsets[lp]; r < task_row_offsets[lp + 1]; ++r) lp_rows[rows[r].kernel_id] = &rows[r];
    const uint64_t h0 = task_offsets[hp], H = task_offsets[hp + 1] - h0;
    const uint64_t l0 = task_offsets[lp], L = task_offsets[lp + 1] - l0;
    std::vector<int64_t> D(L);  // predicted duration of each low-priority kernel
    for (uint64_t j = 0; j < L; ++j) {
      auto it = lp_rows.find(ids[l0 + j]);
      if (it == lp_rows.end()) return UNKNOWN_ID;
      D[j] = predicted(it->second->exec, predictor);
    }
    uint64_t p = 0;     // next low-priority kernel to issue (FIFO)
    int64_t delay = 0;  // accumulated delay of the high-priority task
    const uint64_t g0 = gap_offsets[s];
    for (uint64_t i = 0; i + 1 < H; ++i) {
      auto it = hp_rows.find(ids[h0 + i]);
      if (it == hp_rows.end()) return UNKNOWN_ID;
      const int64_t G = predicted(it->second->gap, predictor);  // predicted idle time
      const int64_t actual = actual_gap_ns[h0 + i];  // idle time that occurred
      if (actual < 0) return INVALID_ARG;
      uint32_t c = 0;
      int64_t f = 0;
      if (G >= min_gap_ns && G >= margin_ns) {
        int64_t r = G - margin_ns;  // remaining predicted idle time
        while (p < L && D[p] <= r) {
          if (feedback && f >= actual) break;  // the next high-priority request is already there
          r -= D[p];
          f += D[p];
          ++p;
          ++c;
        }
        if (f > actual) delay += f - actual;
      }
      fill_count[g0 + i] = c;
      filled_ns[g0 + i] = f;
    }
    if (H > 0) {  // the last launch must be known too, as in oracle_gapfill
      if (hp_rows.find(ids[h0 + H - 1]) == hp_rows.end()) return UNKNOWN_ID;
    }
    hp_delay_ns[s] = delay;
    lp_placed[s] = p;
  }
  return OK;
}


// Gap filling with several low-priority tasks (Algorithm 1 calling Algorithm 2, BestPrioFit).
//
// Scenario s: high-priority task hp_task[s] holds the GPU; its low-priority tasks are the entries
// lp_offsets[s] .. lp_offsets[s+1] of lp_task / lp_prio (priority level 1..9, 1 the highest after the
// high-priority task's own level 0).  Every low-priority task has one waiting request at a time, its
// next kernel; when that is issued, the task's following kernel is enqueued.  For every predicted gap
// that is not skipped (as in oracle_gapfill), with r = gap - margin left:
//   scan the levels from 1 to 9; at the first level that has a waiting request whose predicted
//   duration is <= r, take the one with the longest duration among those (the one closest to r);
//   among equally long ones the one that was enqueued first (the initial requests count as enqueued
//   in the order of the scenario's list); issue it, r -= duration, and scan again from level 1;
//   the gap is done when no level has a request that fits.
// Outputs: per gap the number of kernels issued and their total predicted duration; per
// low-priority entry the number of its kernels issued into gaps and their total predicted duration;
// optionally (issue_offsets[S+1], issue_entry) the entry index (0-based inside the scenario) of every
// issued kernel in issue order.
int oracle_prio_fill(const uint64_t* ids, const uint64_t* task_offsets, uint32_t n_tasks, const void* rows_v,
                     const uint64_t* task_row_offsets, const uint32_t* hp_task, const uint64_t* lp_offsets,
                     const uint32_t* lp_task, const uint32_t* lp_prio, uint64_t n_scenarios, int64_t margin_ns,
                     int64_t min_gap_ns, int predictor, const uint64_t* gap_offsets, uint32_t* fill_count,
                     int64_t* filled_ns, uint64_t* lp_placed, int64_t* lp_placed_ns,
                     const uint64_t* issue_offsets, uint32_t* issue_entry) {
  const Row* rows = static_cast<const Row*>(rows_v);
  if (!task_offsets || !task_row_offsets) return INVALID_ARG;
  if (n_scenarios && (!hp_task || !lp_offsets || !gap_offsets)) return INVALID_ARG;
  if (margin_ns < 0 || min_gap_ns < 0 || predictor < 0 || predictor > 1) return INVALID_ARG;
  if (n_scenarios && lp_offsets[0] != 0) return INVALID_ARG;

  for (uint64_t s = 0; s < n_scenarios; ++s) {
    const uint32_t hp = hp_task[s];
    if (hp >= n_tasks || lp_offsets[s + 1] < lp_offsets[s]) return INVALID_ARG;
    const uint64_t e0 = lp_offsets[s], K = lp_offsets[s + 1] - e0;
    std::map<uint64_t, const Row*> hp_rows;
    for (uint64_t r = task_row_offsets[hp]; r < task_row_offsets[hp + 1]; ++r) hp_rows[rows[r].kernel_id] = &rows[r];

    // the waiting queue of every low-priority task: predicted durations of its kernels, in launch order
    std::vector<std::vector<int64_t>> D(K);
    std::vector<uint64_t> next(K, 0);    // next kernel of task k to issue
    std::vector<uint64_t> stamp(K);      // when the waiting request of task k was enqueued
    for (uint64_t k = 0; k < K; ++k) {
      const uint32_t lp = lp_task[e0 + k];
      if (lp >= n_tasks || lp_prio[e0 + k] < 1 || lp_prio[e0 + k] > 9) return INVALID_ARG;
      std::map<uint64_t, const Row*> lp_rows;
      for (uint64_t r = task_row_offsets[lp]; r < task_row_offsets[lp + 1]; ++r) lp_rows[rows[r].kernel_id] = &rows[r];
      const uint64_t l0 = task_offsets[lp], L = task_offsets[lp + 1] - l0;
      D[k].resize(L);
      for (uint64_t j = 0; j < L; ++j) {
        auto it = lp_rows.find(ids[l0 + j]);
        if (it == lp_rows.end()) return UNKNOWN_ID;
        D[k][j] = predicted(it->second->exec, predictor);
      }
      stamp[k] = k;
      lp_placed[e0 + k] = 0;
      lp_placed_ns[e0 + k] = 0;
    }
    uint64_t clock = K;   // enqueue stamps handed out so far
    uint64_t issued = 0;

    const uint64_t h0 = task_offsets[hp], H = task_offsets[hp + 1] - h0;
    const uint64_t g0 = gap_offsets[s];
    for (uint64_t i = 0; i < H; ++i) {
      auto it = hp_rows.find(ids[h0 + i]);
      if (it == hp_rows.end()) return UNKNOWN_ID;
      if (i + 1 == H) break;  // no gap after the last launch
      const int64_t G = predicted(it->second->gap, predictor);
      uint32_t c = 0;
      int64_t f = 0;
      if (G >= min_gap_ns && G >= margin_ns) {
        int64_t r = G - margin_ns;
        for (;;) {
          // BestPrioFit: the highest level with a request that fits; there the longest; then the oldest
          bool found = false;
          uint64_t best = 0;
          for (uint32_t level = 1; level <= 9 && !found; ++level) {
            for (uint64_t k = 0; k < K; ++k) {
              if (lp_prio[e0 + k] != level || next[k] >= D[k].size()) continue;
              const int64_t d = D[k][next[k]];
              if (d > r) continue;
              if (!found || d > D[best][next[best]] || (d == D[best][next[best]] && stamp[k] < stamp[best])) {
                found = true;
                best = k;
              }
            }
          }
          if (!found) break;
          const int64_t d = D[best][next[best]];
          r -= d;
          f += d;
          ++c;
          ++next[best];
          stamp[best] = clock++;   // the task's following kernel is enqueued now
          lp_placed[e0 + best] += 1;
          lp_placed_ns[e0 + best] += d;
          if (issue_entry) issue_entry[issue_offsets[s] + issued] = static_cast<uint32_t>(best);
          ++issued;
        }
      }
      fill_count[g0 + i] = c;
      filled_ns[g0 + i] = f;
    }
  }
  return OK;
}


// The best partner of every high-priority task among evaluated combinations.
//
// Scenario s pairs hp_task[s] with lp_task[s]; its gap fill left filled_ns for its gaps
// gap_offsets[s] .. gap_offsets[s+1]-1 and the completion time lp_completion_ns[s] of the partner.
// scenario_filled_ns[s] = the idle time of the high-priority task that the partner's kernels fill = the
// sum of the scenario's filled_ns (the high-priority task's idle time is the same in all its scenarios,
// so the largest filled time is also the largest filled fraction).  For every task t that is the
// high-priority task of at least one scenario: the scenario with the largest filled time; among equal
// ones the one whose partner completes earliest; among those the first in scenario order.  Outputs per
// task: that scenario, its partner and its filled time; a task that heads no scenario gets
// best_scenario = 2^64 - 1, best_lp = 2^32 - 1, best_filled_ns = 0.
int oracle_pairing_best(const uint32_t* hp_task, const uint32_t* lp_task, uint64_t n_scenarios, uint32_t n_tasks,
                        const uint64_t* gap_offsets, const int64_t* filled_ns, const int64_t* lp_completion_ns,
                        int64_t* scenario_filled_ns, uint64_t* best_scenario, uint32_t* best_lp,
                        int64_t* best_filled_ns) {
  if (n_scenarios && (!hp_task || !lp_task || !gap_offsets || !lp_completion_ns || !scenario_filled_ns)) return INVALID_ARG;
  if (n_tasks && (!best_scenario || !best_lp || !best_filled_ns)) return INVALID_ARG;
  for (uint32_t t = 0; t < n_tasks; ++t) {
    best_scenario[t] = ~0ull;
    best_lp[t] = ~0u;
    best_filled_ns[t] = 0;
  }
  if (n_scenarios && gap_offsets[0] != 0) return INVALID_ARG;
  for (uint64_t s = 0; s < n_scenarios; ++s) {
    if (hp_task[s] >= n_tasks || lp_task[s] >= n_tasks || gap_offsets[s + 1] < gap_offsets[s]) return INVALID_ARG;
    int64_t total = 0;
    for (uint64_t g = gap_offsets[s]; g < gap_offsets[s + 1]; ++g) total += filled_ns[g];
    scenario_filled_ns[s] = total;
  }
  for (uint64_t s = 0; s < n_scenarios; ++s) {
    const uint32_t t = hp_task[s];
    const uint64_t b = best_scenario[t];
    const bool better = b == ~0ull || scenario_filled_ns[s] > scenario_filled_ns[b] ||
                        (scenario_filled_ns[s] == scenario_filled_ns[b] && lp_completion_ns[s] < lp_completion_ns[b]);
    if (better) {
      best_scenario[t] = s;
      best_lp[t] = lp_task[s];
      best_filled_ns[t] = scenario_filled_ns[s];
    }
  }
  return OK;
}


// Merging the profiles of two sets of runs of the same tasks (Section 3.2: SK_j and SG_j are sums over
// all T runs of a task divided by the number of samples; a run of N kernels has N - 1 idle times, so
// profiling every run on its own and merging keeps the idle time between two runs out of the samples).
//
// a and b hold rows of the same n_tasks tasks (task t: rows a_offsets[t] .. a_offsets[t+1]-1, ordered by
// ID as an unsigned number; likewise b).  Output: per task the union of the IDs, in the same order.  An ID
// in one input only: its row, unchanged.  An ID in both: count and sum add up (sum modulo 2^64), min and
// max combine; these are exactly the values a profile of all samples would have, and so is the mean.
// The percentiles of the union cannot be known from two rows: p50 and p95 are taken, for the execution
// times and for the idle times separately, from the input that has more samples (from a if equal).
int oracle_profile_merge(const void* a_rows_v, const uint64_t* a_offsets, const void* b_rows_v, const uint64_t* b_offsets,
                         uint32_t n_tasks, void* rows_out_v, uint64_t row_capacity, uint64_t* offsets_out,
                         uint64_t* n_rows_out) {
  const Row* a = static_cast<const Row*>(a_rows_v);
  const Row* b = static_cast<const Row*>(b_rows_v);
  Row* out = static_cast<Row*>(rows_out_v);
  if (!a_offsets || !b_offsets || !offsets_out || !n_rows_out) return INVALID_ARG;
  if (a_offsets[0] != 0 || b_offsets[0] != 0) return INVALID_ARG;
  auto merge_stats = [](const Stats& x, const Stats& y) {
    if (x.count == 0) return y;
    if (y.count == 0) return x;
    Stats m;
    m.count = x.count + y.count;
    m.sum = x.sum + y.sum;
    m.min = std::min(x.min, y.min);
    m.max = std::max(x.max, y.max);
    const Stats& larger = y.count > x.count ? y : x;
    m.p50 = larger.p50;
    m.p95 = larger.p95;
    return m;
  };
  uint64_t n = 0;
  for (uint32_t t = 0; t < n_tasks; ++t) {
    if (a_offsets[t + 1] < a_offsets[t] || b_offsets[t + 1] < b_offsets[t]) return INVALID_ARG;
    offsets_out[t] = n;
    std::map<uint64_t, Row> rows;   // ordered by ID
    for (uint64_t r = a_offsets[t]; r < a_offsets[t + 1]; ++r) {
      if (a[r].task != t) return INVALID_ARG;
      if (r > a_offsets[t] && a[r].kernel_id <= a[r - 1].kernel_id) return INVALID_ARG;
      rows[a[r].kernel_id] = a[r];
    }
    for (uint64_t r = b_offsets[t]; r < b_offsets[t + 1]; ++r) {
      if (b[r].task != t) return INVALID_ARG;
      if (r > b_offsets[t] && b[r].kernel_id <= b[r - 1].kernel_id) return INVALID_ARG;
      auto it = rows.find(b[r].kernel_id);
      if (it == rows.end()) {
        rows[b[r].kernel_id] = b[r];
      } else {
        it->second.exec = merge_stats(it->second.exec, b[r].exec);
        it->second.gap = merge_stats(it->second.gap, b[r].gap);
      }
    }
    for (const auto& kv : rows) {
      if (n < row_capacity) {
        Row row;
        std::memset(&row, 0, sizeof(row));
        row.kernel_id = kv.first;
        row.task = t;
        row.exec = kv.second.exec;
        row.gap = kv.second.gap;
        out[n] = row;
      }
      ++n;
    }
  }
  offsets_out[n_tasks] = n;
  *n_rows_out = n;
  return n > row_capacity ? ROW_CAPACITY : OK;
}


}  // extern "C"
