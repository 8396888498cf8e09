/*
 * fikit.h - C ABI of the FIKIT trace-profiling and gap-fill evaluation library (gfx950).
 *
 * The library evaluates, offline and in bulk, two steps of FIKIT (arXiv 2311.10359):
 *
 *   fikit_profile  - the statistical output of the measurement phase (Section 3.2, "Data
 *                    acquisition and statistical output during the measurement phase"): every
 *                    intercepted launch is given its Kernel ID (Section 3.2, "Identifying each
 *                    kernel"), its execution time K and the idle time G up to the next launch
 *                    of the same task are measured from the recorded start/end times, and per
 *                    task and unique ID (the set S_UID) the samples are reduced.  The paper
 *                    keeps the means SK_j and SG_j; a row here carries count and sum (mean =
 *                    sum / count) and also min, max and the nearest-rank 50th and 95th
 *                    percentile of the same samples.
 *
 *   fikit_gapfill  - Algorithm 1 (FIKIT procedure) driven by that table, for one
 *                    high-priority and one low-priority task per scenario: after each
 *                    high-priority kernel the predicted idle time of its ID is looked up, small
 *                    gaps are skipped, and the low-priority task's next kernel is issued for as
 *                    long as its predicted duration does not exceed what is left of the gap
 *                    (Algorithm 2 with a single waiting request is first-in-first-out).
 *
 * Both at once: fikit_profile_gapfill.  Beside these: fikit_measure (the per-launch measurements themselves), fikit_gapfill_replay (the
 * fill replayed against the idle times that occurred, without and with real-time feedback),
 * fikit_prio_fill (several low-priority tasks per scenario in the priority queues of Algorithm 2),
 * fikit_pairing_best (the best partner of every high-priority task among evaluated combinations) and
 * fikit_profile_merge (the profile of further runs merged into the profile so far).
 *
 * Conventions
 *   - d_* arguments are device pointers, h_* are host pointers.  The caller owns every buffer,
 *     including the workspace; the library allocates no device memory and its results depend
 *     on nothing but a call's arguments (the only things it keeps between calls are the
 *     measurement aid fikit_trace_* and the scratch address of fikit_gapfill_static).  Inputs
 *     are left untouched.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the default
 *     stream).  Every call but fikit_gapfill_static synchronises that stream before it returns, so
 *     outputs and the returned status are final on return.
 *   - Return value: FIKIT_OK or a negative fikit_status.  Nothing aborts or throws.  After an
 *     error the contents of the output buffers are unspecified.
 *   - Everything is integer arithmetic (nanoseconds, counts); results are exact.
 *   - Limits: n_records, n_ids < 2^32 - 2^24.  Timestamps must be such that end - start and
 *     next start - end fit in int64, and a task's predicted timeline (sum of p50 values over
 *     its launches) fits in int64.
 */
#ifndef FIKIT_H
#define FIKIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* One intercepted kernel launch.  64 bytes, little endian, 16-byte aligned.
 * Bytes 0..31 are the identity of the kernel (what the Kernel ID is made of); `run` says which
 * of the task's measured runs the launch belongs to (Section 3.2: a task is measured over T runs;
 * a run's launches are consecutive; any numbers will do, only a change from one launch to the
 * next matters); bytes 52..63 are ignored. */
typedef struct fikit_launch {
  uint32_t name_id;      /*  0  interned kernel function name          */
  uint32_t grid[3];      /*  4  grid dimensions x, y, z                */
  uint32_t block[3];     /* 16  block dimensions x, y, z               */
  uint32_t shmem;        /* 28  dynamic shared-memory bytes            */
  int64_t start_ns;      /* 32  device time at which the kernel began  */
  int64_t end_ns;        /* 40  device time at which the kernel ended  */
  uint32_t run;          /* 48  measured run the launch belongs to     */
  uint8_t reserved[12];  /* 52  ignored                                */
} fikit_launch;

/* Statistics of one sample set.  count == 0 implies every other field is 0. */
typedef struct fikit_stats {
  uint64_t count; /* number of samples                                            */
  uint64_t sum;   /* sum of samples modulo 2^64                                   */
  int64_t min;
  int64_t max;
  int64_t p50;    /* nearest rank: the ceil(50*count/100)-th smallest sample     */
  int64_t p95;    /* nearest rank: the ceil(95*count/100)-th smallest sample     */
} fikit_stats;

/* One row of a task's profile: a unique Kernel ID with the statistics of its execution
 * times (exec) and of the idle times that followed its launches (gap).  128 bytes. */
typedef struct fikit_row {
  uint64_t kernel_id;
  uint32_t task;
  uint32_t reserved0;
  fikit_stats exec; /* offset 16 */
  fikit_stats gap;  /* offset 64 */
  uint8_t reserved1[16];
} fikit_row;

typedef enum fikit_status {
  FIKIT_OK = 0,
  FIKIT_INVALID_ARG = -1,         /* NULL or misaligned pointer, offsets not monotone or not ending
                                     at the element count, task index out of range, size limit  */
  FIKIT_WORKSPACE_TOO_SMALL = -2,
  FIKIT_ROW_CAPACITY = -3,        /* more rows than row_capacity; *h_n_rows holds the need       */
  FIKIT_BAD_RECORD = -4,          /* some record has end_ns < start_ns                          */
  FIKIT_UNKNOWN_ID = -5,          /* a scenario launch whose ID is absent from its task's rows  */
  FIKIT_HIP_ERROR = -6,           /* the HIP runtime reported an error, or a bounded wait ran out
                                     (fikit_set_wait_limit)                                      */
  FIKIT_UNSUPPORTED = -7,         /* fikit_prio_fill: a scenario whose list entries and launches
                                     together number 2^32 or more                                 */
  FIKIT_TOO_LARGE = -8            /* fikit_gapfill_static: more launches or tasks than its built-in
                                     scratch buffer holds                                          */
} fikit_status;

/* Bytes of device workspace fikit_profile needs for these sizes (0 on size overflow). */
size_t fikit_profile_workspace_bytes(uint64_t n_records, uint32_t n_tasks);

/*
 * Measurement-phase statistics (Section 3.2).
 *
 *   d_records          [n_records] launches; task t owns records
 *                      d_task_offsets[t] .. d_task_offsets[t+1]-1, in launch order.
 *   d_task_offsets     [n_tasks+1] uint64, non-decreasing, first 0, last n_records.
 *   d_ids_out          [n_records] receives every launch's Kernel ID in launch order: the
 *                      64-bit FNV-1a hash of record bytes 0..31.  May be NULL.
 *   d_rows_out         [row_capacity] receives the rows, ordered by task, then by kernel_id as
 *                      an unsigned number.  Execution time of a launch = end_ns - start_ns; the
 *                      idle time after a launch = max(0, next start_ns - end_ns), where "next"
 *                      is the following launch of the same task and run; the last launch of a run
 *                      has none (a run of N launches gives N - 1 idle times, Section 3.2), so the
 *                      rows of a trace that holds several runs are exactly the statistics over all
 *                      of them, percentiles included.
 *   d_task_row_offsets [n_tasks+1] receives, per task, where its rows start (last = row count).
 *   h_n_rows           host; receives the number of rows (also on FIKIT_ROW_CAPACITY).
 *   d_workspace        256-byte aligned, at least fikit_profile_workspace_bytes(...) bytes.
 *
 * Errors: INVALID_ARG, WORKSPACE_TOO_SMALL, ROW_CAPACITY, BAD_RECORD, HIP_ERROR.
 * n_records == 0 yields zero rows and FIKIT_OK.
 */
int fikit_profile(const fikit_launch* d_records, uint64_t n_records,
                  const uint64_t* d_task_offsets, uint32_t n_tasks, uint64_t* d_ids_out,
                  fikit_row* d_rows_out, uint64_t row_capacity, uint64_t* d_task_row_offsets,
                  uint64_t* h_n_rows, void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Where a launch's predicted execution / idle time is read in its ID's row. */
typedef enum fikit_predictor {
  FIKIT_PREDICT_P50 = 0,  /* nearest-rank median of the ID's samples                              */
  FIKIT_PREDICT_MEAN = 1  /* their mean, SK_j / SG_j of Section 3.2: sum / count, rounded down
                             to whole nanoseconds (0 if the ID has no sample)                     */
} fikit_predictor;

typedef struct fikit_gapfill_params {
  int64_t margin_ns;  /* reserved at the end of every gap; a gap shorter than this is skipped */
  int64_t min_gap_ns; /* gaps predicted shorter than this are skipped (Algorithm 1)           */
  int32_t predictor;  /* a fikit_predictor                                                     */
  int32_t reserved;   /* must be 0                                                             */
} fikit_gapfill_params;

/* Bytes of device workspace fikit_gapfill needs for these sizes (0 on size overflow). */
size_t fikit_gapfill_workspace_bytes(uint64_t n_ids, uint32_t n_tasks, uint64_t n_scenarios);

/*
 * Gap filling (Algorithm 1, with Algorithm 2 reduced to one waiting request).
 *
 *   d_ids, d_task_offsets, n_tasks   Kernel IDs of every launch of every task, laid out as in
 *                      fikit_profile (its d_ids_out and d_task_offsets).
 *   d_rows, d_task_row_offsets       the profile of those tasks (fikit_profile's outputs).
 *   d_hp_task, d_lp_task [n_scenarios] the high- and the low-priority task of each scenario.
 *   h_params           host pointer.  margin_ns, min_gap_ns >= 0.
 *   d_gap_offsets      [n_scenarios+1] where each scenario's per-gap outputs start; scenario s
 *                      with H launches in its high-priority trace owns max(H-1, 0) slots.
 *   d_fill_count, d_filled_ns  per gap: low-priority kernels issued into it, and the sum of
 *                      their predicted durations.
 *   d_lp_completion_ns [n_scenarios] predicted time at which the low-priority task ends, on a
 *                      timeline that starts at 0 with the first high-priority kernel and on
 *                      which high-priority kernels are never delayed; low-priority kernels
 *                      that found no gap run back to back after the last high-priority kernel.
 *   d_lp_placed        [n_scenarios] number of low-priority kernels issued into gaps.
 *
 * Predicted execution time of a launch = exec.p50 of its ID's row; predicted idle time after a
 * high-priority launch = gap.p50 of its ID's row (or the means, see fikit_predictor).  A gap is skipped if its prediction is below
 * min_gap_ns or below margin_ns; otherwise gap - margin_ns nanoseconds may be filled.
 *
 * Errors: INVALID_ARG, WORKSPACE_TOO_SMALL, UNKNOWN_ID, HIP_ERROR.
 */
int fikit_gapfill(const uint64_t* d_ids, const uint64_t* d_task_offsets, uint32_t n_tasks,
                  const fikit_row* d_rows, const uint64_t* d_task_row_offsets,
                  const uint32_t* d_hp_task, const uint32_t* d_lp_task, uint64_t n_scenarios,
                  const fikit_gapfill_params* h_params, const uint64_t* d_gap_offsets,
                  uint32_t* d_fill_count, int64_t* d_filled_ns, int64_t* d_lp_completion_ns,
                  uint64_t* d_lp_placed, void* d_workspace, size_t workspace_bytes,
                  void* hip_stream);

/* Bytes of device workspace fikit_profile_gapfill needs for these sizes (0 on size overflow). */
size_t fikit_profile_gapfill_workspace_bytes(uint64_t n_records, uint32_t n_tasks, uint64_t n_scenarios);

/*
 * fikit_profile followed by fikit_gapfill on the same traces, as one call: the measurement-phase statistics
 * (Section 3.2) and Algorithm 1 driven by them.  Arguments and outputs are those of the two calls (d_ids_out is
 * required here; the profile's outputs are the gap fill's inputs), and every output equals what the two calls give
 * one after the other.  The difference is inside: a task that one workgroup profiles whole has its launches'
 * predicted durations and idle times written by that workgroup while the launches are still in its registers, so
 * the gap fill need not read the Kernel IDs again and look every one up (with at least 4096 scenarios and
 * predictions below 2^32 - 1 ns; otherwise, and for the tasks that take other paths, exactly the kernels of the two
 * calls run).
 *
 *   d_workspace   256-byte aligned, at least fikit_profile_gapfill_workspace_bytes(...) bytes.
 *
 * Errors: those of fikit_profile (after which the gap fill is not attempted) and of fikit_gapfill.
 */
int fikit_profile_gapfill(const fikit_launch* d_records, uint64_t n_records, const uint64_t* d_task_offsets,
                          uint32_t n_tasks, uint64_t* d_ids_out, fikit_row* d_rows_out, uint64_t row_capacity,
                          uint64_t* d_task_row_offsets, uint64_t* h_n_rows, const uint32_t* d_hp_task,
                          const uint32_t* d_lp_task, uint64_t n_scenarios, const fikit_gapfill_params* h_params,
                          const uint64_t* d_gap_offsets, uint32_t* d_fill_count, int64_t* d_filled_ns,
                          int64_t* d_lp_completion_ns, uint64_t* d_lp_placed, void* d_workspace,
                          size_t workspace_bytes, void* hip_stream);

/* Largest inputs of fikit_gapfill_static. */
#define FIKIT_STATIC_MAX_IDS (1u << 20)   /* launches of all tasks together */
#define FIKIT_STATIC_MAX_TASKS 16384u

/*
 * fikit_gapfill for callers that cannot allocate device memory or wait for the device: code that is being
 * captured into a HIP graph, tight serving loops, harnesses that forbid hipMalloc.  It computes what
 * fikit_gapfill computes, with these differences:
 *
 *   - no workspace argument: the library's own scratch buffer is used, a device array of about 24 MiB that is
 *     part of the library's code object (every GPU the library is used on holds one for the life of the
 *     process).  Inputs beyond FIKIT_STATIC_MAX_IDS launches or FIKIT_STATIC_MAX_TASKS tasks are refused with
 *     FIKIT_TOO_LARGE before anything is enqueued.
 *   - n_ids (= d_task_offsets[n_tasks]) and n_gaps (= d_gap_offsets[n_scenarios]) are passed by the caller
 *     instead of being read back; a mismatch is reported as FIKIT_INVALID_ARG through d_status.
 *   - the call only enqueues work on hip_stream and returns; it does not synchronise.  d_status (device,
 *     int32) receives the fikit_status of the data-dependent checks (FIKIT_OK, FIKIT_INVALID_ARG,
 *     FIKIT_UNKNOWN_ID) once the stream has run that far; outputs are valid only if it is FIKIT_OK.  The
 *     return value covers what the host can see: INVALID_ARG, TOO_LARGE, HIP_ERROR.
 *   - it calls no hipMalloc / hipFree, records no events and creates nothing; the first call on a device
 *     looks up that device's scratch address and sets one kernel attribute.
 *
 * All calls on one GPU share that GPU's scratch buffer: calls that may overlap in time (different streams,
 * different threads) race and must be serialised by the caller.  Calls on one stream are safe back to back.
 */
int fikit_gapfill_static(const uint64_t* d_ids, uint64_t n_ids, const uint64_t* d_task_offsets, uint32_t n_tasks,
                         const fikit_row* d_rows, const uint64_t* d_task_row_offsets,
                         const uint32_t* d_hp_task, const uint32_t* d_lp_task, uint64_t n_scenarios,
                         const fikit_gapfill_params* h_params, const uint64_t* d_gap_offsets, uint64_t n_gaps,
                         uint32_t* d_fill_count, int64_t* d_filled_ns, int64_t* d_lp_completion_ns,
                         uint64_t* d_lp_placed, int32_t* d_status, void* hip_stream);

/* Bytes of device workspace fikit_measure needs. */
size_t fikit_measure_workspace_bytes(void);

/*
 * The two per-launch measurements of Section 3.2 ("Measuring the execution and idle time of
 * kernel"), as they stand in the trace.
 *
 *   d_records, d_task_offsets, n_tasks   as in fikit_profile.
 *   d_exec_ns   [n_records] receives end_ns - start_ns of every launch.
 *   d_gap_ns    [n_records] receives the idle time after the launch, max(0, start_ns of the
 *               task's next launch - end_ns), or -1 for the last launch of a run or task.
 *   d_workspace 256-byte aligned, at least fikit_measure_workspace_bytes() bytes.
 *
 * Buffers are the caller's; the call synchronises the stream.  Errors: INVALID_ARG,
 * WORKSPACE_TOO_SMALL, BAD_RECORD, HIP_ERROR.
 */
int fikit_measure(const fikit_launch* d_records, uint64_t n_records, const uint64_t* d_task_offsets,
                  uint32_t n_tasks, int64_t* d_exec_ns, int64_t* d_gap_ns, void* d_workspace,
                  size_t workspace_bytes, void* hip_stream);

typedef struct fikit_replay_params {
  int64_t margin_ns;   /* as in fikit_gapfill_params                                            */
  int64_t min_gap_ns;  /* as in fikit_gapfill_params                                            */
  int32_t feedback;    /* 0: profile-only controller; non-zero: real-time feedback             */
  int32_t predictor;   /* a fikit_predictor                                                     */
} fikit_replay_params;

/* Bytes of device workspace fikit_gapfill_replay needs for these sizes (0 on size overflow). */
size_t fikit_replay_workspace_bytes(uint64_t n_ids, uint32_t n_tasks, uint64_t n_scenarios);

/*
 * The gap filling of fikit_gapfill replayed against the idle times that actually occurred (the
 * paragraph "Real time feedback to stop error propagation" of the paper's scheduling section,
 * Figure "Runtime Feedback").  Decisions are taken on predictions exactly as in fikit_gapfill;
 * issued kernels run back to back from the start of the gap for their predicted duration.
 *
 *   d_actual_gap_ns  [n_ids] idle time that followed every launch (fikit_measure's d_gap_ns);
 *                    only high-priority launches but the trace's last are looked at, and theirs
 *                    must be >= 0 (else INVALID_ARG: a high-priority trace that holds several
 *                    measured runs has no idle time at the run ends and cannot be replayed).
 *   h_params         host pointer.  feedback == 0: every kernel that fits the predicted gap is
 *                    issued (the paper's profile-only controller).  feedback != 0: before each
 *                    issue the controller checks whether the next high-priority request has
 *                    arrived, i.e. whether the time already filled in this gap has reached the
 *                    actual idle time, and if so issues nothing more into this gap.
 *   d_fill_count, d_filled_ns  per gap, as in fikit_gapfill (with feedback == 0 they equal its).
 *   d_hp_delay_ns    [n_scenarios] sum over the scenario's gaps of max(0, filled - actual idle
 *                    time): what the high-priority task is delayed by (the paper's overhead 1
 *                    without feedback, overhead 2 with it).  Every gap is charged on its own;
 *                    later launches of the trace are not shifted.
 *   d_lp_placed      [n_scenarios] number of low-priority kernels issued into gaps.
 *   all other arguments as in fikit_gapfill.
 *
 * Predictions of 2^32 - 1 ns (about 4.29 s) or more are handled by slower 64-bit kernels.
 * Errors: INVALID_ARG, WORKSPACE_TOO_SMALL, UNKNOWN_ID, HIP_ERROR.
 */
int fikit_gapfill_replay(const uint64_t* d_ids, const uint64_t* d_task_offsets, uint32_t n_tasks,
                         const fikit_row* d_rows, const uint64_t* d_task_row_offsets,
                         const int64_t* d_actual_gap_ns, const uint32_t* d_hp_task,
                         const uint32_t* d_lp_task, uint64_t n_scenarios,
                         const fikit_replay_params* h_params, const uint64_t* d_gap_offsets,
                         uint32_t* d_fill_count, int64_t* d_filled_ns, int64_t* d_hp_delay_ns,
                         uint64_t* d_lp_placed, void* d_workspace, size_t workspace_bytes,
                         void* hip_stream);

/* Most low-priority tasks of a scenario that fikit_prio_fill's fast kernels take (a scenario may hold more). */
#define FIKIT_PRIO_MAX_LP 64

/* Bytes of device workspace fikit_prio_fill needs for these sizes (0 on size overflow). */
size_t fikit_prio_fill_workspace_bytes(uint64_t n_ids, uint32_t n_tasks, uint64_t n_scenarios);

/*
 * Gap filling with several low-priority tasks per scenario: Algorithm 1 calling the whole of
 * Algorithm 2 (BestPrioFit) over the priority queues Q1..Q9 (Q0 is the high-priority task that
 * holds the GPU).
 *
 *   d_lp_offsets [n_scenarios+1] uint64, first 0, non-decreasing: scenario s owns the entries
 *                d_lp_offsets[s] .. d_lp_offsets[s+1]-1 of d_lp_task / d_lp_prio; the entries of a
 *                scenario and their launches together must number fewer than 2^32 (else
 *                FIKIT_UNSUPPORTED).
 *   d_lp_task    per entry, a low-priority task of the scenario (a task may appear in several
 *                entries and scenarios; every entry is a separate run of it).
 *   d_lp_prio    per entry, its priority level, 1 (highest) .. 9 (else FIKIT_INVALID_ARG).
 *   d_fill_count, d_filled_ns  per gap (laid out by d_gap_offsets as in fikit_gapfill): kernels
 *                issued into it and the sum of their predicted durations.
 *   d_lp_placed, d_lp_placed_ns  per entry: how many of its kernels were issued into gaps, and
 *                the sum of their predicted durations.
 *   all other arguments as in fikit_gapfill.
 *
 * Every low-priority task has one waiting request at a time, its next kernel; when that is issued
 * its following kernel is enqueued.  In every gap that is not skipped (the rule of fikit_gapfill),
 * with r = gap - margin_ns left: the levels are scanned from 1 to 9; at the first level that holds
 * a request whose predicted duration is at most r, the longest such request is taken (among equally
 * long ones the one enqueued first; the initial requests count as enqueued in list order), issued,
 * r is reduced by its duration and the scan starts again at level 1; the gap is done when no level
 * holds a request that fits.  With one entry per scenario the per-gap results are fikit_gapfill's.
 *
 * If some scenario holds more than FIKIT_PRIO_MAX_LP low-priority tasks, or a prediction is 2^32 - 1 ns or more,
 * slower kernels do the call (one lane per scenario, every decision looks at all its waiting requests).
 * Errors: INVALID_ARG, WORKSPACE_TOO_SMALL, UNKNOWN_ID, UNSUPPORTED, HIP_ERROR.
 */
int fikit_prio_fill(const uint64_t* d_ids, const uint64_t* d_task_offsets, uint32_t n_tasks,
                    const fikit_row* d_rows, const uint64_t* d_task_row_offsets,
                    const uint32_t* d_hp_task, const uint64_t* d_lp_offsets,
                    const uint32_t* d_lp_task, const uint32_t* d_lp_prio, uint64_t n_scenarios,
                    const fikit_gapfill_params* h_params, const uint64_t* d_gap_offsets,
                    uint32_t* d_fill_count, int64_t* d_filled_ns, uint64_t* d_lp_placed,
                    int64_t* d_lp_placed_ns, void* d_workspace, size_t workspace_bytes,
                    void* hip_stream);

/* Bytes of device workspace fikit_pairing_best needs (0 on size overflow). */
size_t fikit_pairing_workspace_bytes(uint32_t n_tasks);

/*
 * Which low-priority partner suits each high-priority task best, among combinations that have been
 * evaluated with fikit_gapfill (the paper's discussion section, "What Tasks are Suitable for Sharing a
 * GPU": measure combinations beforehand, then look a task's best matching partner up).
 *
 *   d_hp_task, d_lp_task [n_scenarios]  the combinations (any number per task, in any order).
 *   d_gap_offsets, d_filled_ns, d_lp_completion_ns   fikit_gapfill's layout and outputs for them.
 *   d_scenario_filled_ns [n_scenarios] receives the idle time of the high-priority task that the
 *                      partner's kernels fill: the sum of the scenario's d_filled_ns (modulo 2^64).
 *   d_best_scenario, d_best_lp, d_best_filled_ns [n_tasks]  per task t that is the high-priority task of
 *                      at least one scenario: the scenario with the largest filled time (= the largest
 *                      filled fraction, the task's idle time being the same in all its scenarios); among
 *                      equal ones the one whose partner completes earliest; among those the first in
 *                      scenario order; its partner; its filled time.  Other tasks get 2^64 - 1,
 *                      2^32 - 1 and 0.
 *   d_workspace        256-byte aligned, at least fikit_pairing_workspace_bytes(n_tasks) bytes.
 *
 * Buffers are the caller's; the call synchronises the stream.
 * Errors: INVALID_ARG (also: task index out of range, gap offsets not monotone),
 * WORKSPACE_TOO_SMALL, HIP_ERROR.
 */
int fikit_pairing_best(const uint32_t* d_hp_task, const uint32_t* d_lp_task, uint64_t n_scenarios,
                       uint32_t n_tasks, const uint64_t* d_gap_offsets, const int64_t* d_filled_ns,
                       const int64_t* d_lp_completion_ns, int64_t* d_scenario_filled_ns,
                       uint64_t* d_best_scenario, uint32_t* d_best_lp, int64_t* d_best_filled_ns,
                       void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of device workspace fikit_profile_merge needs (0 on size overflow). */
size_t fikit_profile_merge_workspace_bytes(uint32_t n_tasks);

/*
 * Merges the profile of further runs of the same tasks into the profile of the runs so far (Section
 * 3.2: the statistics run over all T measured runs of a task, and a run of N kernels contributes N - 1
 * idle times; profiling every run on its own and merging keeps the idle time between runs out).
 *
 *   d_rows_a, d_task_row_offsets_a   a profile as fikit_profile writes it: task t owns rows
 *                      d_task_row_offsets_a[t] .. [t+1]-1, ordered by kernel_id as an unsigned number,
 *                      each with task == t (else FIKIT_INVALID_ARG).
 *   d_rows_b, d_task_row_offsets_b   another profile of the same n_tasks tasks.
 *   d_rows_out         [row_capacity] receives, per task, one row per ID of either input, in the same
 *                      order.  An ID of one input only: its row.  An ID of both: count and sum add up
 *                      (sum modulo 2^64), min and max combine: exactly the values a profile of all
 *                      samples together would hold, and so is the mean (FIKIT_PREDICT_MEAN).  The
 *                      percentiles of the union cannot be known from two rows: p50 and p95 are taken,
 *                      for exec and for gap separately, from the input whose block has more samples
 *                      (from a if equal).
 *   d_task_row_offsets_out [n_tasks+1], h_n_rows   as in fikit_profile (also on FIKIT_ROW_CAPACITY).
 *   d_workspace        256-byte aligned, at least fikit_profile_merge_workspace_bytes(n_tasks) bytes.
 *
 * The output must not overlap the inputs.  Buffers are the caller's; the call synchronises the stream.
 * Errors: INVALID_ARG, WORKSPACE_TOO_SMALL, ROW_CAPACITY, HIP_ERROR.
 */
int fikit_profile_merge(const fikit_row* d_rows_a, const uint64_t* d_task_row_offsets_a,
                        const fikit_row* d_rows_b, const uint64_t* d_task_row_offsets_b, uint32_t n_tasks,
                        fikit_row* d_rows_out, uint64_t row_capacity, uint64_t* d_task_row_offsets_out,
                        uint64_t* h_n_rows, void* d_workspace, size_t workspace_bytes, void* hip_stream);

const char* fikit_status_string(int status);
int fikit_version(void);

/*
 * Bounded waits.  The sort that fikit_profile falls back on for tasks with too many distinct Kernel IDs lets a tile of
 * a task wait for what the task's earlier tiles publish (statistical result 1 of Section 3.2 is the grouping this sort
 * performs).  Every such wait is bounded: after `polls` fruitless polls of one word (default 2^24, seconds) the tile
 * gives up, nothing is written outside the task, every kernel still ends, and the call returns FIKIT_HIP_ERROR instead
 * of hanging.  fikit_set_wait_limit sets the bound for later calls (0 restores the default); a tiny bound makes the
 * failure path testable from the host.  Process-wide, not thread safe.
 */
void fikit_set_wait_limit(uint32_t polls);

/*
 * Per-kernel timing, a measurement aid (off by default; process-wide, not thread safe).
 * fikit_trace_enable(1) clears the table and makes every later fikit_profile / fikit_gapfill
 * call record a HIP event on its stream before each kernel launch; when the call ends, the time
 * between consecutive events is added to the entry named after the launch that opened the
 * interval ("host_sync" entries hold the time the host spent reading a count back).
 * fikit_trace_read returns the number of entries and, for 0 <= index < that number, stores the
 * entry's name (a static string), its accumulated milliseconds and its number of intervals;
 * any of the three output pointers may be NULL.
 */
void fikit_trace_enable(int on);
int fikit_trace_read(int index, const char** name, double* total_ms, int* launches);

#ifdef __cplusplus
}
#endif
#endif /* FIKIT_H */
