/*
 * daris.h -- C ABI of the MI355X DARIS hot path.
 *
 * DARIS (Sec. III-IV of the paper) runs several periodic, two-priority DNN inference tasks concurrently on
 * partitions ("contexts") of one GPU.  A task's DNN is cut into sequential stages; a synchronisation point
 * at every stage boundary is the only preemption / migration point (Sec. III-B1).  Here a partition is a set
 * of compute units: a CU mask plus N_s CU-masked hardware queues ("streams") that the library creates and feeds
 * itself; the sum of partition sizes may exceed the 256 CUs of the device (oversubscription, Sec. III-C2).
 *
 * General rules
 *   - Every function returns a status (0 = DARIS_OK, negative = error) or a non-negative handle; nothing
 *     throws or aborts.  daris_last_error() gives the text of the calling thread's last failure.
 *   - All calls come from one API thread.  The library runs one internal scheduler thread in real-time mode.
 *   - "host" pointers are ordinary CPU memory, read during the call only (the library copies what it keeps).
 *     "device" pointers are HIP device memory owned by the caller, which must stay valid until the job that
 *     uses them has completed (daris_run_until_idle() or the blocking run calls return).  The library's kernels run
 *     on queues of its own, not on a HIP stream: what the caller's streams wrote into an input buffer must be
 *     complete (stream or device synchronised) before the job is released, and logits are complete and visible
 *     to every HIP stream once the job has completed.  daris_task_set_io and daris_forward synchronise the device
 *     themselves; daris_release_job, the hot path, does not.
 *   - Times are int64 nanoseconds.  In virtual-time mode they are positions on the library's virtual clock;
 *     in real-time mode they count from the library's epoch (set by daris_commit()).
 *   - Utilisations (eq. 3-7) are evaluated in Q32 fixed point: u = floor(mret * 2^32 / T).
 */
#ifndef DARIS_H
#define DARIS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t daris_status;
typedef int32_t daris_part; /* partition handle: 0,1,2,... in creation order; <0 is an error code */
typedef int32_t daris_task; /* task handle:      0,1,2,... in registration order; <0 is an error code */

enum {
  DARIS_OK = 0,
  DARIS_EINVAL = -1, /* bad argument / unsupported layer shape */
  DARIS_ENOMEM = -2, /* host or device allocation failed */
  DARIS_EHIP = -3,   /* a HIP or HSA runtime call failed (text in daris_last_error) */
  DARIS_ESTATE = -4, /* call not allowed in the current state (e.g. not initialised, already committed) */
  DARIS_ERANGE = -5  /* handle or index out of range */
};

/* daris_init flags */
enum {
  DARIS_VIRTUAL_TIME = 1,     /* decisions run on a virtual clock fed by daris_set_virtual_time tables        */
  DARIS_NO_DEVICE = 2,        /* host logic only: no HIP call is made, no kernel runs (needs VIRTUAL_TIME)     */
  DARIS_NO_LAST = 4,          /* ablation (Sec. VI, "No Last"): last stages get no extra level                 */
  DARIS_NO_PRIOR = 8,         /* ablation ("No Prior"): a missed predecessor gives no extra level              */
  DARIS_NO_FIXED = 16,        /* ablation ("No Fixed"): all stages share one level, EDF only                   */
  DARIS_HP_ADMISSION = 32,    /* Overload+HPA (Sec. VI-I): HP jobs must pass the test in their own context     */
  DARIS_KEEP_ACTIVATIONS = 64, /* debugging: one buffer per layer output so daris_read_layer (daris_debug.h) works */
  DARIS_WAVE_PRIORITY = 128,  /* the convolution waves of high-priority tasks raise their issue priority on the CU:
                                 where partitions overlap, HP stages run faster and LP stages slower (measured:
                                 HP response -5 %, LP +12 %, aggregate throughput -2 %); off by default          */
  DARIS_SHARED_QUEUE = 256,   /* the N_s streams of a partition feed ONE hardware queue instead of one each: their
                                 stages execute one after the other, but the next one is already queued when a
                                 stage ends, so the host round trip of the boundary is hidden.  For GPUs on which
                                 only a few hardware queues make progress at a time; scheduling decisions (and the
                                 trace) are those of N_s streams; off by default                                */
  DARIS_NO_PAIR = 512,        /* tasks registered under this flag launch a residual block's shortcut convolution and
                                 first convolution separately instead of in one two-problem launch (A/B and tests)  */
  DARIS_NO_FUSED_INGEST = 1024, /* ... and convert the input layout in a launch of its own instead of inside the first
                                 convolution                                                                     */
  DARIS_NO_STAGED_ROWS = 2048, /* ... and feed every convolution's pixel operand straight from global memory to registers
                                 instead of fetching whole 64-byte rows through LDS where the shape allows (A/B)   */
  DARIS_NO_SMALL_TILES = 4096, /* ... and keep 32-pixel tiles with a K split across workgroups (and its reduction launch)
                                 for deep layers of few pixels, instead of 16-pixel tiles (A/B)                  */
  DARIS_NO_FUSED_DW = 8192     /* ... and run a 3x3 depthwise convolution in a launch of its own instead of computing it
                                 inside the 1x1 convolution that is its only reader (A/B and tests)              */
};

enum { DARIS_LP = 0, DARIS_HP = 1 };
enum { DARIS_FP32 = 0, DARIS_BF16 = 1 };
enum { DARIS_OP_CONV = 0, DARIS_OP_MAXPOOL = 1, DARIS_OP_GAVGPOOL = 2, DARIS_OP_FC = 3 };
enum { DARIS_ACT_NONE = 0, DARIS_ACT_RELU = 1, DARIS_ACT_RELU6 = 2 };

/* Outcome of daris_release_job (Sec. IV-B1). */
enum {
  DARIS_ACCEPTED = 1,         /* admitted in the task's current partition                                      */
  DARIS_MIGRATED = 2,         /* admitted after migration to another partition (LP only)                       */
  DARIS_REJECT_ADMISSION = 3, /* failed eq. (12) in every partition                                            */
  DARIS_REJECT_OVERRUN = 4,   /* LP: the task's previous job is still active                                   */
  DARIS_QUEUED = 5            /* HP: waits behind the task's previous job, starts when it ends                 */
};

/*
 * One layer of a DNN.  Layer l reads the output of layer in_from (-1 = the network input) and, if
 * res_from >= 0, adds the output of layer res_from (same shape as its own output) before the activation.
 *   CONV     : cross-correlation, zero padding, groups == 1 (dense) or groups == c_in == c_out (depthwise);
 *              w = host float[c_out][c_in/groups][k][k], b = host float[c_out] or NULL.  BN must already be
 *              folded into (w, b).  c_in and c_out must be multiples of 4 (8 for bf16 tasks) except that the
 *              network input may have 1..4 channels.
 *   MAXPOOL  : k x k window, padding acts as -inf.  w, b unused.
 *   GAVGPOOL : mean over all pixels.  w, b unused.
 *   FC       : w = host float[c_out][c_in], c_in = C*H*W of the producing tensor flattened in (c, y, x)
 *              order; b as for CONV.
 */
typedef struct daris_layer {
  int32_t op;
  int32_t c_in, c_out;
  int32_t k, stride, pad;
  int32_t groups;
  int32_t act;
  int32_t in_from;
  int32_t res_from;
  const float* w;
  const float* b;
} daris_layer;

/* A DNN: input tensor (c, h, w), fp32 NCHW in caller memory; arithmetic type of the task. */
typedef struct daris_dnn {
  int32_t n_layers;
  int32_t in_c, in_h, in_w;
  int32_t dtype; /* DARIS_FP32: fp32 storage, fp32 MFMA.  DARIS_BF16: bf16 weights/activations, fp32 accumulate */
  const daris_layer* layers;
} daris_dnn;

typedef struct daris_task_stats {
  int64_t released, accepted, completed, missed; /* DMR = missed / accepted (Sec. V)                         */
  int64_t rejected_admission, rejected_overrun;
  int64_t resp_min_ns, resp_max_ns, resp_sum_ns; /* response time = completion - release                     */
  int64_t first_release_ns, last_finish_ns;
  int32_t partition;                            /* ctx_i: current partition                                  */
  int32_t n_stages;
} daris_task_stats;

/* 32-byte little-endian trace record; `type` values follow. */
typedef struct daris_trace_rec {
  uint64_t seq;
  int64_t t_ns;
  uint8_t type, level, stage, partition;
  uint16_t task, stream;
  uint32_t job;
  uint32_t aux; /* DISPATCH: virtual deadline - release; STAGE_DONE/JOB_DONE: 1 = (virtual) deadline missed;
                   REJECT: 1 admission, 2 overrun; MIGRATE: source partition, +256 if forced; ACCEPT: 1 if the job
                   had been queued */
} daris_trace_rec;
enum {
  DARIS_T_RELEASE = 1, DARIS_T_ACCEPT = 2, DARIS_T_REJECT = 3, DARIS_T_MIGRATE = 4, DARIS_T_DISPATCH = 5,
  DARIS_T_STAGE_DONE = 6, DARIS_T_JOB_DONE = 7, DARIS_T_QUEUED = 8, DARIS_T_CMD_MIGRATE = 9
};

/* ---- life cycle ------------------------------------------------------------------------------------------ */

/* Select HIP device `device` and reset all library state.  `seed` is stored for reproducibility reports only
 * (the scheduler draws no random numbers).  Returns DARIS_ESTATE if already initialised.  The first call with a
 * device loads the kernels onto it; they stay there until the process ends, and later calls must name the same device. */
daris_status daris_init(int device, uint64_t seed, int flags);
/* Wait for running work, stop the worker threads, free every queue, signal and device buffer. */
daris_status daris_shutdown(void);
const char* daris_last_error(void);
/* Bound, in nanoseconds (> 0, default 20 s, process-wide, kept across daris_init), on every wait of the host for the GPU: a
 * stage boundary, a direct execution, room in a queue.  When it expires -- or when the runtime reports an error on a queue
 * -- the call that waited returns DARIS_EHIP (a scheduled run: daris_run_until_idle and the blocking run calls do), and
 * because the state of the GPU work is unknown from then on, every later call except daris_shutdown, daris_last_error and
 * the read-only accessors returns DARIS_EHIP too.  daris_shutdown then lets the queues run dry for at most 5 s each before
 * it frees the buffers. */
daris_status daris_set_timeout(int64_t ns);
/* The partition size (CUs, 8..256; default 128, reset by daris_init) that the launch plans of tasks registered from now on
 * are balanced for: how many workgroups a convolution is cut into, so that a launch fills the CUs in whole rounds.  A
 * task's plan is fixed when it is registered and is the same wherever its stages run, so its results never depend on the
 * partition (Sec. III-A: a task may be migrated to any context).  A set-up with equal partitions of another size calls
 * this with that size (ResNet-18 on 64-CU partitions: 273 us with plans for 128 CUs, 243 us with plans for 64); with
 * unequal partitions a plan for the smaller ones costs as much on the larger ones as it gains. */
daris_status daris_set_plan_cus(int n_cu);

/* ---- partitions (Sec. III-C) ------------------------------------------------------------------------------- */

/* N_SM = ceil_even(OS * N_max / N_c) with OS = os_num/os_den (Sec. III-C2); pure integer helper, needs no init. */
int32_t daris_cu_per_partition(int32_t os_num, int32_t os_den, int32_t n_cu_max, int32_t n_c);
/* New partition of n_cu compute units (1..256) with one stream.  Partition p covers the logical CUs
 * [start_p, start_p + n_cu) mod 256 with start_p = sum of earlier sizes mod 256, so partitions overlap only when
 * their sizes sum past 256 (oversubscription).  Must precede daris_commit(). */
daris_part daris_create_partition(int n_cu);
/* Number of streams N_s of a partition (1..8); each stream runs one stage at a time (Sec. III-C1). */
daris_status daris_partition_set_streams(daris_part p, int n_s);
/* Copy the partition's CU mask (8 x 32 bits, bit i of word i/32 = logical CU i). */
daris_status daris_partition_get_mask(daris_part p, uint32_t mask_out[8]);

/* ---- tasks (Sec. III-A) ------------------------------------------------------------------------------------ */

/* Register a periodic task: copies and re-packs the weights into device memory, allocates activation buffers.
 * period_ns = T_i > 0, deadline_ns = D_i > 0 (the paper uses D_i = T_i), priority DARIS_HP or DARIS_LP.
 * The task starts with one stage; its partition is chosen by daris_commit() (Algorithm 1). */
daris_task daris_register_task(const daris_dnn* dnn, int64_t period_ns, int64_t deadline_ns, int priority);
/* Cut the DNN into k sequential stages (Sec. III-B1).  A cut is legal after layer l when no later layer reads
 * anything produced before l except l's own output.  The k-1 cuts minimise the largest per-stage MAC count; ties
 * go to the lexicographically smallest cut list.  DARIS_ERANGE if k > legal cuts + 1. */
daris_status daris_split_stages(daris_task t, int k);
/* Writes the index of the first layer of each stage into first_layer[0..cap) and returns the stage count. */
int32_t daris_get_stage_cuts(daris_task t, int32_t* first_layer, int32_t cap);
/* Per-stage AFET (Sec. IV-A1), ns > 0: the execution-time estimate used until the stage has run once. */
daris_status daris_set_afet(daris_task t, int stage, int64_t ns);
/* MRET window size ws (eq. 1), default 5. */
daris_status daris_set_window(int ws);
/* Virtual-time mode: execution time of jobs job_lo..job_hi-1 of (task, stage) when run in partition p;
 * et_ns = host int64[job_hi - job_lo], each >= 1. */
daris_status daris_set_virtual_time(daris_task t, int stage, daris_part p, int64_t job_lo, int64_t job_hi,
                                    const int64_t* et_ns);
/* Offline phase (Algorithm 1): HP tasks, then LP tasks, each in registration order, go to the partition of least
 * total utilisation afet_i/T_i (ties: lowest index).  Creates the CU-masked streams, starts the real-time
 * clock and the scheduler thread.  Called implicitly by the first release. */
daris_status daris_commit(void);
/* Current partition ctx_i of a task (after commit). */
daris_part daris_get_partition(daris_task t);

/* ---- online phase (Sec. IV-B) ------------------------------------------------------------------------------ */

/* Release one job of task t.  d_input = device float[c][h][w]; d_logits = device float[n_out] receiving the last
 * layer's output in (c, y, x) order.  release_ns: virtual-time mode -- the release instant, non-decreasing over
 * calls (events before it are simulated first; stage completions at exactly release_ns are processed before the
 * release, dispatching at release_ns happens after all releases of that instant); real-time mode -- the nominal
 * release used for deadlines and response times, or -1 for "now".  *decision (may be NULL) receives a
 * DARIS_ACCEPTED.. code.  LP jobs take the admission test eq. (11)-(12); HP jobs are always scheduled. */
daris_status daris_release_job(daris_task t, const void* d_input, void* d_logits, int64_t release_ns,
                               int32_t* decision);
/* Forced migration of task t to partition p: applied at once unless a stage of t is running, else at that
 * stage's boundary; later jobs of t stay in p. */
daris_status daris_migrate(daris_task t, daris_part p);
/* Virtual time: simulate until no event is left.  Real time: block until no job is active or queued. */
daris_status daris_run_until_idle(void);

/* Per-task I/O pool for the library-driven runs below: job m reads input (m mod n_inputs) of d_inputs =
 * device float[n_inputs][c*h*w] and writes logits row (m mod n_slots) of d_logits = device float[n_slots][n_out].
 * The kernel arguments that name these buffers are prepared here, once per buffer, in device memory.
 * DARIS_ESTATE while a job of the task is active. */
daris_status daris_task_set_io(daris_task t, const void* d_inputs, int32_t n_inputs, void* d_logits, int32_t n_slots);
/* Release job m of task i at phase_ns[i] + m * T_i for m < n_jobs[i] (arrays indexed by task handle, host), in
 * (time, task) order, and return when every job has finished or was rejected. */
daris_status daris_run_periodic(const int64_t* phase_ns, const int32_t* n_jobs);
/* Saturated variant: every task with n_jobs[i] > 0 releases its next job the instant the previous one finishes
 * (or is rejected) until n_jobs[i] were released or, if total_jobs > 0, until total_jobs were released over all
 * tasks together (tasks in faster partitions then contribute more jobs).  Real-time mode only. */
daris_status daris_run_closed_loop(const int32_t* n_jobs, int64_t total_jobs);

/* ---- observation ------------------------------------------------------------------------------------------- */

daris_status daris_get_stats(daris_task t, daris_task_stats* out);
/* Copies up to cap_bytes / 32 not-yet-read trace records into buf (host), releases them, and returns the byte count
 * copied.  A trace nobody reads is capped at 4 Mi records: the older half is dropped (seq numbers show the gap). */
int64_t daris_trace_read(void* buf, int64_t cap_bytes);
/* Current MRET of a stage (eq. 1), ns. */
int64_t daris_get_mret(daris_task t, int stage);

/* ---- direct execution and calibration (instrumentation lives in daris_debug.h) --------------------------------- */

/* Run the whole DNN of task t once, stage after stage, on stream 0 of partition p, and wait for it.  No scheduler
 * state is touched.  The logits do not depend on p or on the stage split. */
daris_status daris_forward(daris_task t, const void* d_input, void* d_logits, daris_part p);
/* daris_forward for callers that cannot allocate device memory: code that runs while another part of the process
 * captures a HIP graph, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels in the same
 * order, hence bit-identical logits; but the task's activation tensors and split-K partial sums live in a static device
 * array of 16 MiB that the library's device image brings along (every GPU the library was initialised on holds its own
 * copy until the process ends) instead of the buffers allocated at registration, and every launch's argument block goes
 * through the queue's ring of host-visible memory.  The call allocates nothing: no hipMalloc / hipFree, no pinned memory,
 * no queue or signal; the first call for a task encodes that task's launches against the array in ordinary host memory.
 *   - The streams must exist already (daris_commit, or any execution, came first: creating them allocates);
 *     DARIS_ESTATE otherwise.
 *   - The task's activation slots plus workspace must fit the array (every configured network but VGG-16 does);
 *     DARIS_ERANGE otherwise, with both sizes in daris_last_error().
 *   - All calls on a GPU share that GPU's array, which keeps whatever the last call left in it.  Nothing in it has to be
 *     cleared: every kernel reads only what an earlier kernel of the same call wrote.  Two calls that overlapped on one
 *     GPU would race on it; the library runs them one at a time.  Weights stay where registration put them. */
daris_status daris_forward_static(daris_task t, const void* d_input, void* d_logits, daris_part p);
/* Measure per-stage execution times of task t alone on partition p (`reps` runs, the maximum is kept) and store
 * them as the task's AFET values. */
daris_status daris_calibrate_afet(daris_task t, daris_part p, int reps);

/* Average full-load execution time (Sec. IV-A1): like daris_calibrate_afet, but while every other stream of every
 * partition runs one forward pass of a distinct other task drawn with the generator seeded by daris_init's seed;
 * the per-stage averages over `reps` runs become the task's AFET values.  Call while no job is active. */
daris_status daris_calibrate_afet_loaded(daris_task t, daris_part p, int reps);
#ifdef __cplusplus
}
#endif
#endif /* DARIS_H */
