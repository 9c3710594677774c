/*
 * gcaps_rta — batched schedulability testing of real-time tasksets on one
 * AMD Instinct MI355X (gfx950), C ABI.
 *
 * For every taskset of a batch the library computes the worst-case
 * response-time bound R_i of every task (Eq. 1: R_i = C_i + G_i + I^C_i + I^G_i)
 * under
 *   - GCAPS preemptive priority-based GPU context scheduling (Sec. 5.3,
 *     Lemmas 8-15), and/or
 *   - the default round-robin time-sliced TSG scheduling of the driver
 *     (Sec. 5.2, Eq. 3, Lemmas 1-7),
 * in busy-waiting or self-suspension mode, as the least fixed point of the
 * respective recurrence, tasks taken in decreasing priority, and the verdict
 * "every R_i <= D_i" (the response-time test of Sec. 4.3 / Sec. 6.1).
 *
 * Task model (Sec. 3): a taskset has n sporadic tasks with fixed priorities and
 * constrained deadlines, each bound to one CPU core.  Task tau_i has C_i (sum of
 * its CPU segments), period T_i, deadline D_i <= T_i, priority pi_i, eta^g_i GPU
 * segments G_{i,j} = (G^m_{i,j}, G^e_{i,j}): CPU-side launch/driver work and pure
 * GPU work (copies, kernels).  G_i is taken as sum_j (G^m_{i,j} + G^e_{i,j}).
 * Per taskset: theta (GPU context-switch overhead, Def. 1), epsilon (runlist
 * update delay, Def. 2) and the TSG time slice L (Eq. 3).
 *
 * All times are unsigned integer microseconds.  All arithmetic is exact
 * integer arithmetic; results do not depend on launch shape or batch order.
 *
 * Where the lemmas as printed leave a choice, the library computes one reading
 * only (there is no switch for another one):
 *   - G_i := sum_j (G^m_{i,j} + G^e_{i,j}) (Sec. 3 bounds G_i from above only); under
 *     GCAPS the task's own 2 * epsilon * eta^g_i (Sec. 5.3) is added to Eq. 1;
 *   - Lemma 10: the sum over the GPU-using higher-priority tasks of tau_i's core is
 *     applied to every tau_i; the printed guard eta^g_i > 0 would let a CPU-only task
 *     ignore the busy-waiting of a task above it on its core;
 *   - Lemma 7: the jitter J^c_h is applied to self-suspending (GPU-using) tau_h only,
 *     as Lemma 15 does; CPU-only tasksets then reduce to the classic analysis;
 *   - Lemma 8: B^C_i = (eta^g_i + 1) * epsilon for every task, GPU-using or not;
 *   - Lemma 4: the set is the GPU-using tasks outside hpp(tau_i) plus tau_h itself;
 *   - Lemma 11 is applied as printed, with no condition on tau_i's core.
 *
 * What a verdict of 1 means: every bound R_i of the lemmas, under these readings, is
 * at most D_i.  Two effects that a concrete schedule (gcaps_simulate_batch) shows are
 * charged by no lemma, so a simulated job can respond later than R_i:
 *   - round-robin, theta > 0: Eq. 3 counts theta + L per time slice of every other
 *     TSG and nothing for the switch that brings in the task's own slice; a segment
 *     of k slices can see up to k more theta than Eq. 3 holds.  With theta = 0, or
 *     in a schedule that leaves those switches out, no simulated job was seen above
 *     its bound;
 *   - GCAPS, epsilon > 0: gcapsGpuSegEnd() is a system call of the task's own thread
 *     (Sec. 4.2), so a task that is preempted on its core after its GPU work keeps its
 *     TSGs on the runlist until it runs again, and lower-priority GPU segments wait
 *     for that long; Lemmas 10 and 13 charge tau_h's GPU segment and its updates, not
 *     this wait.  Tasks for which every GPU-using task of higher priority is the
 *     highest-priority task of its core cannot be reached by it.
 *
 * Plain C, no exceptions, no callbacks.  Every function returns GCAPS_OK (0) or
 * a negative error code and never aborts.  A context is not thread-safe: use
 * one context per host thread.
 */
#ifndef GCAPS_RTA_H
#define GCAPS_RTA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gcaps_ctx gcaps_ctx; /* opaque: device id, stream, device scratch */

/*
 * One batch of tasksets of identical shape.  All pointers of one batch are
 * either host pointers (gcaps_rta_batch) or device pointers on the context's
 * device (gcaps_rta_batch_device).  The caller owns every buffer for the
 * duration of the call (for the device entry point: until the work queued on
 * the context's stream has completed); the library neither frees nor keeps them.
 *
 * Layout: per-taskset arrays have n_tasksets elements; per-task arrays are
 * [n_tasksets][n_tasks] row-major, tasks in caller order (any priority order);
 * per-segment arrays are [n_tasksets][n_tasks][max_gseg] row-major.  Every array needs the alignment of its
 * element type and no more (the outputs likewise: 8 bytes for the response times); arrays may be views into larger
 * buffers.
 */
typedef struct {
  uint32_t n_tasksets; /* >= 1 */
  uint32_t n_tasks;    /* n, 1..255, the same for every taskset of the batch */
  uint32_t max_gseg;   /* S, 0..255: GPU-segment slots per task */
  /* per taskset */
  const uint32_t *theta_us; /* theta: context-switch overhead of round-robin TSG scheduling (Def. 1) */
  const uint32_t *eps_us;   /* epsilon = alpha + theta: runlist update delay of GCAPS (Def. 2) */
  const uint32_t *slice_us; /* L >= 1: TSG time slice (Eq. 3) */
  /* per task */
  const uint32_t *cpu_us;      /* C_i (Sec. 3) */
  const uint8_t *n_cseg;       /* eta^c_i; part of the task tuple, used by no bound; may be NULL */
  const uint32_t *period_us;   /* T_i >= 1 */
  const uint32_t *deadline_us; /* 1 <= D_i <= T_i */
  const int32_t *prio;         /* pi_i: larger = higher; equal values: lower caller index ranks higher */
  const uint8_t *core;         /* CPU core of tau_i (partitioned scheduling) */
  const uint8_t *n_gseg;       /* eta^g_i <= S; 0 = CPU-only task */
  /* per segment; slots j >= eta^g_i are ignored; both may be NULL when S = 0 */
  const uint32_t *gm_us; /* G^m_{i,j} */
  const uint32_t *ge_us; /* G^e_{i,j} */
} gcaps_batch;

/* which analysis */
enum { GCAPS_POLICY_GCAPS = 1, GCAPS_POLICY_RR = 2, GCAPS_POLICY_BOTH = 3 };
enum { GCAPS_WAIT_BUSY = 0, GCAPS_WAIT_SUSPEND = 1 };

/* error codes */
enum {
  GCAPS_OK = 0,
  GCAPS_EINVAL = -1,  /* null pointer, zero or out-of-range size, unknown selector */
  GCAPS_ETASK = -2,   /* a taskset violates the task model: T = 0, D = 0, D > T, L = 0, eta^g > S
                         (gcaps_gprio_rta_batch: or its GPU priorities disagree with prio on a core) */
  GCAPS_ENOMEM = -3,  /* host or device allocation failed */
  GCAPS_EDEVICE = -4, /* a HIP call failed (no device, launch failure, ...) */
  GCAPS_ESIZE = -5    /* the call needs more device scratch than it may take now: a call that the stream is
                         recording into a HIP graph and that is larger than every direct call made before it
                         (nothing is freed or allocated; make a direct call of these sizes first), or a batch
                         beyond the limits of gcaps_rta_batch_device_static */
};

/* response-time sentinels in out_resp */
#define GCAPS_RESP_MISS (-1)         /* first task in priority order whose bound exceeds D_i */
#define GCAPS_RESP_NOT_ANALYSED (-2) /* every lower-priority task of that taskset */

/*
 * Creates a context on device `device_id`.  `hip_stream` is a hipStream_t on
 * that device on which all work of the context is queued, or NULL for the
 * device's default stream; the stream stays owned by the caller.
 *
 * Tuning knobs are read from the environment here; results never depend on them:
 *   GCAPS_SCREEN_TASKS    tasks per taskset that the first launch analyses (default 4)
 *   GCAPS_DEEP_LANES      lanes per taskset in the second launch, 4 (default) or 8
 *   GCAPS_CHUNK_TASKSETS  cap on the tasksets per internal chunk of a call
 *   GCAPS_DEEP_KERNEL     "lds": the second launch of the analysis keeps its term records in LDS for every
 *                         shape (default: in registers for shapes of at most 32 tasks)
 *   GCAPS_GEN_KERNEL      "taskset": gcaps_taskgen_device with one lane per taskset (default: one lane per task)
 *   GCAPS_GPRIO_KERNEL    "list": the priority search as two launches, the second packing sixteen searched
 *                         tasksets per wavefront (faster when most tasksets are searched deeply; default: one
 *                         pass in which a wavefront reads, searches and answers 16 consecutive tasksets)
 */
int gcaps_create(gcaps_ctx **out, int device_id, void *hip_stream);

/* Waits for the context's queued work, frees its device scratch.  NULL is allowed. */
void gcaps_destroy(gcaps_ctx *ctx);

/*
 * Host-to-host entry point.  `batch` holds HOST pointers.  Copies the batch to
 * the device, runs the analysis there, copies the results back, and returns
 * when they are in place.
 *   policy     GCAPS_POLICY_GCAPS, _RR or _BOTH;  npol = number of policies selected
 *   wait_mode  GCAPS_WAIT_BUSY or GCAPS_WAIT_SUSPEND (applies to every selected policy)
 *   out_resp   host int64 [npol][n_tasksets][n_tasks], tasks in caller order: R_i in
 *              microseconds, or a sentinel.  Policies are stored in increasing
 *              selector value (GCAPS before round-robin).
 *   out_sched  host uint8 [npol][n_tasksets]: 1 iff every task met R_i <= D_i (what the bounds
 *              cover and what they leave out: head of this file)
 *   first_bad_taskset  may be NULL; on GCAPS_ETASK receives the smallest index of
 *              an invalid taskset
 * On any error no output element is defined.
 */
int gcaps_rta_batch(gcaps_ctx *ctx, const gcaps_batch *batch, int policy, int wait_mode,
                    int64_t *out_resp, uint8_t *out_sched, uint32_t *first_bad_taskset);

/*
 * Device-resident entry point: every pointer in `batch`, d_out_resp and
 * d_out_sched is a DEVICE pointer on the context's device, with the layouts
 * above.  The work is queued on the context's stream and the call returns
 * without waiting for it.  Argument errors are reported at once; task-model
 * violations are detected on the device and reported by gcaps_status().
 * Outputs of an invalid taskset are undefined, all others are complete.
 * The launches of a call may be recorded into a HIP graph (stream capture) once a direct call with
 * the same sizes has been made on the context: that call makes the device allocations, a recorded
 * one makes none (GCAPS_ESIZE when it would have to).  A direct call that needs more scratch than any before
 * it frees and reallocates the context's buffers: graphs recorded earlier on this context then point
 * to freed memory and must be recorded again.  A recorded call depends on no earlier call and can be
 * replayed any number of times, with direct calls in between.  The same holds for the other device-resident entry points
 * (gcaps_gprio_assign_batch_device, gcaps_gprio_rta_batch_device, gcaps_simulate_batch_device).
 */
int gcaps_rta_batch_device(gcaps_ctx *ctx, const gcaps_batch *batch, int policy, int wait_mode,
                           int64_t *d_out_resp, uint8_t *d_out_sched);

/*
 * gcaps_rta_batch_device for callers that cannot allocate device memory when they call: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * launches, same results; the scratch of the launches (per-call status words, the hand-over lists
 * between the launches, the columns of the 64-bit kernel: about 14 MiB) is a fixed array that
 * every GPU the library runs on holds until the process ends, so the call allocates and frees
 * nothing, whatever was called before it on the context.
 * Limits: n_tasksets <= 65536 and n_tasks <= 32, else GCAPS_ESIZE (nothing is queued).
 * The array is shared by every call of this function on one GPU, from any context: calls that
 * overlap in time on one GPU race; calls queued on one stream, or otherwise ordered, do not.  The
 * words that must start at zero are cleared by a kernel at the head of each call.  gcaps_status
 * and gcaps_last_wide_count report on it like on gcaps_rta_batch_device.
 */
int gcaps_rta_batch_device_static(gcaps_ctx *ctx, const gcaps_batch *batch, int policy, int wait_mode,
                                  int64_t *d_out_resp, uint8_t *d_out_sched);

/*
 * Waits for the context's stream and reports on the most recent device-resident
 * call (gcaps_rta_batch_device, gcaps_gprio_assign_batch_device): GCAPS_OK, or GCAPS_ETASK with the smallest
 * invalid taskset index in *first_bad_taskset (may be NULL), or GCAPS_EDEVICE.
 */
int gcaps_status(gcaps_ctx *ctx, uint32_t *first_bad_taskset);

/*
 * Diagnostics of the most recent gcaps_rta_batch_device / gcaps_rta_batch call
 * (waits for the stream): how many of its tasksets had numbers outside the
 * 24-bit fast kernel's range and were analysed by the general 64-bit kernel
 * instead.  Results are exact on both routes; the count only explains speed.
 */
int gcaps_last_wide_count(gcaps_ctx *ctx, uint32_t *count);

/*
 * GPU-segment priority assignment (Sec. 4.3) with the analysis of Sec. 5.4, under GCAPS.
 *
 * For every taskset of the batch the library searches GPU-segment priorities pi^g_i by
 * Audsley's scheme: levels are handed out from the lowest (1) to the highest (n); at each
 * level the tasks without a level yet are tried from the lowest to the highest CPU priority
 * (`prio`); a task is a candidate only if no such task of its core has a lower CPU priority
 * (on a core the GPU order must agree with the CPU order, or the taskset may deadlock); the
 * first candidate whose response-time bound meets its deadline takes the level.  The bound
 * of a candidate is that of Sec. 5.3 with the changes of Sec. 5.4: the sums over
 * higher-priority tasks of OTHER cores (second sums of Lemmas 10 and 13, Lemma 11) run over
 * the tasks that would be above it on the GPU, i.e. every other task without a level; the
 * same-core sums are unchanged; every release jitter uses D_h in place of R_h.  The search
 * fails when a level finds no task, or when some task's own demand
 * C_i + G_i + 2*eps*eta^g_i + (eta^g_i + 1)*eps exceeds D_i (it then passes at no level).
 * theta_us and slice_us of the batch are not read (may be NULL here).
 *
 *   wait_mode  GCAPS_WAIT_BUSY or GCAPS_WAIT_SUSPEND
 *   skip       uint8 [n_tasksets] or NULL: tasksets with skip[s] != 0 are not searched
 *              (typically out_sched of the GCAPS analysis: Sec. 6.1 tries separate
 *              priorities only for tasksets that fail with pi^g = pi^c)
 *   out_gprio  int32 [n_tasksets][n_tasks], caller order: level of tau_i, larger = higher
 *              GPU priority; 0 for every task of a taskset that failed or was skipped
 *   out_resp   int64 [n_tasksets][n_tasks]: the bound of tau_i at its level;
 *              GCAPS_RESP_NOT_ANALYSED for a taskset that failed or was skipped
 *   out_sched  uint8 [n_tasksets]: 1 = an assignment was found, or skipped; 0 = none exists
 *
 * gcaps_gprio_assign_batch takes HOST pointers and returns when the results are in place
 * (errors as gcaps_rta_batch); gcaps_gprio_assign_batch_device takes DEVICE pointers, queues
 * the work on the context's stream and returns (errors as gcaps_rta_batch_device;
 * gcaps_status and gcaps_last_wide_count report on it likewise).
 */
int gcaps_gprio_assign_batch(gcaps_ctx *ctx, const gcaps_batch *batch, int wait_mode, const uint8_t *skip,
                             int32_t *out_gprio, int64_t *out_resp, uint8_t *out_sched,
                             uint32_t *first_bad_taskset);
int gcaps_gprio_assign_batch_device(gcaps_ctx *ctx, const gcaps_batch *batch, int wait_mode,
                                    const uint8_t *d_skip, int32_t *d_out_gprio, int64_t *d_out_resp,
                                    uint8_t *d_out_sched);

/*
 * The analysis of Sec. 5.4 for GPU-segment priorities GIVEN by the caller, under GCAPS: the bound
 * of every task with the sums over higher-priority tasks of other cores (second sums of Lemmas 10
 * and 13, Lemma 11) taken over the tasks with a higher GPU priority, and D_h in place of R_h in
 * every jitter (not taken below zero).  The tasks do not depend on each other's bounds: every task
 * is analysed.
 *   gprio      int32 [n_tasksets][n_tasks], caller order: larger = higher GPU priority; equal
 *              values are ordered by CPU priority.  Two tasks of one core ordered differently by
 *              prio and gprio make the taskset invalid (Sec. 4.3: such an order may deadlock);
 *              it is reported like a task-model violation (GCAPS_ETASK, smallest index)
 *   out_resp   int64 [n_tasksets][n_tasks]: R_i, or GCAPS_RESP_MISS where the bound exceeds D_i
 *   out_sched  uint8 [n_tasksets]: 1 iff no task missed
 * Up to 32 tasks per taskset run in a quad-lane 24-bit kernel (tasksets whose numbers leave its range are
 * handed to the general 64-bit kernel, as gcaps_last_wide_count reports); results are exact on both routes.
 * Host / device variants and error reporting as for gcaps_gprio_assign_batch[_device].
 */
int gcaps_gprio_rta_batch(gcaps_ctx *ctx, const gcaps_batch *batch, int wait_mode, const int32_t *gprio,
                          int64_t *out_resp, uint8_t *out_sched, uint32_t *first_bad_taskset);
int gcaps_gprio_rta_batch_device(gcaps_ctx *ctx, const gcaps_batch *batch, int wait_mode, const int32_t *d_gprio,
                                 int64_t *d_out_resp, uint8_t *d_out_sched);

/*
 * Schedule simulation (the observed response times that Sec. 6.2 and Table 5 set against the bounds of Sec. 5):
 * every taskset of the batch is run as a concrete schedule from time 0 to `horizon` (one time unit = one
 * unit of the batch's values) and the largest response time of each task is reported.
 * The system that is simulated (Sec. 2, Sec. 3, Sec. 4.1-4.2, Alg. 1):
 *   - partitioned, fully preemptive fixed-priority CPUs; prio as in the analysis (larger = higher; equal
 *     values: lower caller index first);
 *   - a job of tau_i is eta^g_i + 1 CPU segments around its eta^g_i GPU segments; C_i is dealt to the CPU
 *     segments as evenly as integers allow, the first C_i mod (eta^g_i + 1) of them one unit longer; GPU segment
 *     j is G^m_{i,j} of CPU work, then G^e_{i,j} of GPU work during which the task keeps its core
 *     (GCAPS_WAIT_BUSY; it can be preempted there) or leaves it (GCAPS_WAIT_SUSPEND);
 *   - GCAPS_POLICY_RR: the tasks with outstanding GPU work form a FIFO ring; the head runs for at most L, then,
 *     if another waits, goes to the tail after a switch of theta; a switch also follows a completed segment
 *     when another task waits;
 *   - GCAPS_POLICY_GCAPS: the GPU work of a segment lies between two runlist updates decided as in Alg. 1; an
 *     update that changes the running TSGs takes eps on the caller's core under the driver lock (not
 *     preemptible; the lock goes to the highest-priority requester that holds its core; a requester without
 *     the lock sleeps on it in either waiting mode, Sec. 5.3 naming it an rt-mutex, and the lower-priority
 *     tasks of its core run meanwhile), one that only joins or leaves the pending list takes no time; only the task whose TSGs are running makes GPU progress;
 *   - releases are strictly periodic: tau_i at offset_i, offset_i + T_i, ...; deadline_us is not used and
 *     may be NULL;
 *   - events of one instant take effect in decreasing priority, so results do not depend on caller order.
 *   offset     uint32 [n_tasksets][n_tasks] first releases, or NULL: all released at 0
 *   gprio      int32 [n_tasksets][n_tasks] priorities of the GPU segments (Sec. 4.3; e.g. out_gprio of
 *              gcaps_gprio_assign_batch), or NULL: the task priorities.  The runlist decisions of
 *              GCAPS_POLICY_GCAPS compare these (larger = higher; among equal values the higher task priority
 *              is served first); CPU scheduling and the driver lock go by prio
 *   policy     GCAPS_POLICY_*; BOTH: two output planes, GCAPS then round-robin
 *   horizon    1..2^31: length of the simulated interval
 *   out_mort   int64 [P][n_tasksets][n_tasks]: largest response time among the jobs that completed
 *              within the horizon, 0 when none did
 *   out_jobs   uint32 [P][n_tasksets][n_tasks]: number of those jobs
 *   out_flag   uint8 [P][n_tasksets]: 1 when a job was released while its predecessor was still running; the
 *              simulation of that taskset stops there and its outputs hold what had completed until then
 * Limits: n_tasks <= 32 (else GCAPS_EINVAL); a taskset with T = 0, L = 0, eta^g > S or a core index >= 64
 * makes the call fail with GCAPS_ETASK (smallest index; outputs unspecified).
 * One lane simulates one taskset under one policy and jumps from event to event (end of a segment, slice,
 * switch or update; a release).  gcaps_simulate_batch takes HOST pointers and returns when the results are in
 * place; gcaps_simulate_batch_device takes DEVICE pointers, queues the work on the context's stream and
 * returns (errors as gcaps_rta_batch_device; gcaps_status reports on it likewise).
 */
int gcaps_simulate_batch(gcaps_ctx *ctx, const gcaps_batch *batch, const uint32_t *offset, const int32_t *gprio,
                         int policy, int wait_mode, uint32_t horizon, int64_t *out_mort, uint32_t *out_jobs,
                         uint8_t *out_flag, uint32_t *first_bad_taskset);
int gcaps_simulate_batch_device(gcaps_ctx *ctx, const gcaps_batch *batch, const uint32_t *d_offset,
                                const int32_t *d_gprio, int policy, int wait_mode, uint32_t horizon,
                                int64_t *d_out_mort, uint32_t *d_out_jobs, uint8_t *d_out_flag);

/*
 * Synthetic input generated on the device (the evaluation of Sec. 6.1 analyses streams of randomly generated
 * tasksets; generating a batch where it is analysed saves the host-to-device copy).  The recipe is that of the
 * host generator of this package: per core a utilisation drawn from [util_lo, util_hi] and split over the
 * tasks of the core by UUniFast; per task a log-uniform period in [period_lo, period_hi] (D = T), eta^g in
 * [eta_lo, eta_hi], C + G = u T, the share G / (C + G) drawn from [share_lo, share_hi] and dealt evenly to the
 * segments, each half G^m and half G^e; theta = eps drawn from [overhead_lo, overhead_hi]; L = slice_us;
 * rate-monotonic priorities over the taskset; tasks i*tasks_per_core .. on core i.  Taskset k of the call uses
 * the random stream (seed, stream, first_index + k): a batch can be generated in pieces and regenerated.
 * The *_fixed members, if not NULL, are DEVICE arrays [n_tasksets] that fix a value per taskset instead of
 * drawing it.  The batch is the host generator's bit for bit: integer random streams, IEEE double operations in
 * one fixed order without fused multiply-add, and the generator's own logarithm and power routines on both sides.
 * A CPU-only task (eta^g = 0 drawn) keeps its whole demand u T as CPU time.
 * batch: sizes and DEVICE pointers of the buffers to fill (n_tasks must equal n_cores * tasks_per_core, eta_hi
 * <= max_gseg; n_cseg is ignored); the call queues one kernel on the context's stream and returns.
 * Errors: GCAPS_EINVAL for null pointers or inconsistent ranges, GCAPS_EDEVICE.
 */
typedef struct {
  uint64_t seed, stream, first_index;
  uint32_t n_cores, tasks_per_core;
  double util_lo, util_hi;
  const double *util_fixed;
  uint32_t eta_lo, eta_hi;
  double share_lo, share_hi;
  const double *share_fixed;
  uint32_t period_lo, period_hi;
  uint32_t overhead_lo, overhead_hi;
  const uint32_t *overhead_fixed;
  uint32_t slice_us;
  const uint32_t *slice_fixed;
} gcaps_taskgen_spec;

int gcaps_taskgen_device(gcaps_ctx *ctx, const gcaps_taskgen_spec *spec, const gcaps_batch *batch);

/*
 * The generation recipe of the schedulability experiments on the device (Sec. 6.1, Table 3): per CPU a number
 * of tasks drawn from [per_cpu_lo, per_cpu_hi] and a utilisation drawn from [util_lo, util_hi], split over the
 * tasks by UUniFast; periods uniform in [period_lo, period_hi] (D = T); round(ratio n) tasks, ratio drawn from
 * [gpu_ratio_lo, gpu_ratio_hi] and the tasks chosen at random, use the GPU with eta^g in [eta_lo, eta_hi]
 * segments; C + G = u T; G / C drawn from [gc_lo, gc_hi]; G dealt evenly to the segments and each segment split
 * by G^m / G drawn from [gm_lo, gm_hi] (whole microseconds, G^e >= 1); rate-monotonic priorities; tasks
 * re-allocated to the CPUs by worst-fit decreasing (by utilisation, ties by index; at most 8 CPUs).  theta,
 * epsilon and L are constants.  Taskset k of the stream (seed, stream, first_index + k) is the one the host
 * generator of this package produces for the same parameters, bit for bit.
 *
 * Tasksets differ in their number of tasks; a batch holds tasksets of one count:
 *   gcaps_table3_count_device     writes the task count of tasksets 0 .. n_tasksets-1 to d_n_tasks (DEVICE,
 *                                 uint32 [n_tasksets]);
 *   gcaps_table3_generate_device  fills `batch` (sizes and DEVICE pointers as for gcaps_taskgen_device;
 *                                 max_gseg >= eta_hi): row r is taskset d_index[r] (DEVICE, uint32
 *                                 [batch->n_tasksets]; NULL: taskset r), which must have batch->n_tasks tasks.
 *                                 A taskset of another count leaves its row unwritten and makes gcaps_status
 *                                 report GCAPS_ETASK with the smallest such row.
 * Both queue one kernel on the context's stream and return.  Errors: GCAPS_EINVAL (null pointers,
 * inconsistent ranges, more than 8 CPUs, more than 255 tasks), GCAPS_EDEVICE.
 */
typedef struct {
  uint64_t seed, stream, first_index;
  uint32_t n_cpus, per_cpu_lo, per_cpu_hi;
  double gpu_ratio_lo, gpu_ratio_hi;
  double util_lo, util_hi;
  uint32_t period_lo, period_hi;
  uint32_t eta_lo, eta_hi;
  double gc_lo, gc_hi;
  double gm_lo, gm_hi;
  uint32_t theta_us, eps_us, slice_us;
} gcaps_table3_spec;

int gcaps_table3_count_device(gcaps_ctx *ctx, const gcaps_table3_spec *spec, uint32_t n_tasksets, uint32_t *d_n_tasks);
int gcaps_table3_generate_device(gcaps_ctx *ctx, const gcaps_table3_spec *spec, const uint32_t *d_index,
                                 const gcaps_batch *batch);

/*
 * Diagnostics of the most recent gcaps_simulate_batch[_device] call (waits for the stream): the number of
 * steps its lanes took in total, a step being one jump to the next event of a taskset's schedule (Sec. 6.2
 * defines no such count; it measures the work of the simulation).
 */
int gcaps_last_sim_steps(gcaps_ctx *ctx, uint64_t *steps);

/*
 * Optional ordering (off by default) of the tasksets that need the second,
 * full-depth launch: a counting sort by how close to its deadline the last task
 * analysed in the first launch comes (R_k / D_k, 256 buckets, most slack first),
 * so that long walks start early and the tasksets sharing a wavefront stop at
 * similar ranks.  Results are identical either way; only the time differs: 1-4 %
 * faster where few tasksets reach the second launch, much slower where most do
 * (the positions inside a bucket come from one counter per bucket).
 * enable: 0 or 1.
 */
int gcaps_set_binning(gcaps_ctx *ctx, int enable);

/*
 * Continue-after-miss (off by default) for gcaps_rta_batch / gcaps_rta_batch_device: the analysis
 * of a taskset goes on below a task whose bound exceeds its deadline.  The response time of that
 * task is unknown, so the jitters J^c_h, J^g_h of the tasks below it take D_h in place of R_h
 * (proof of Lemma 10; a jitter is not taken below zero).  Every task is analysed: out_resp holds
 * R_i or GCAPS_RESP_MISS and never GCAPS_RESP_NOT_ANALYSED; out_sched is unchanged.  Nothing can be
 * settled from the highest-priority tasks alone in this mode: expect several times the run time.
 * enable: 0 or 1.
 */
int gcaps_set_continue_after_miss(gcaps_ctx *ctx, int enable);

/*
 * Measured integer VALU rates of the context's device: the denominator of the fraction of the 32-bit
 * integer VALU peak that the metric of this library's benchmark names (no passage of the paper: it never
 * times its analysis).  For each instruction kind a kernel of independent dependency chains of that one
 * instruction, eight wavefronts per SIMD, is timed with events on the context's stream (the call waits for
 * the stream, allocates a few KB of device memory for the duration of the call and frees it).
 *   lane_ops_per_s[k]  lane-operations per second of kind k (a wavefront instruction = 64; multiply-add = 1);
 *                      GCAPS_PROBE_TERM is the four-instruction sequence of one interference term
 *                      ceil((R + J) / T) * cost of the fast kernels (add, mul_hi_u24, shift, mad_u24),
 *                      counted as four lane-operations
 *   cu_count, clock_khz, wavefront_size, simd_per_cu   as the HIP runtime reports them for the device
 *   spec_lane_ops_per_s   cu_count * simd_per_cu * 16 lanes * clock: one full-rate 32-bit operation per
 *                      lane and cycle
 * Errors: GCAPS_EINVAL, GCAPS_ENOMEM, GCAPS_EDEVICE.
 */
enum {
  GCAPS_PROBE_ADD_U32 = 0,
  GCAPS_PROBE_MAD_U32_U24 = 1,
  GCAPS_PROBE_MUL_HI_U32_U24 = 2,
  GCAPS_PROBE_MUL_LO_U32 = 3,
  GCAPS_PROBE_MUL_HI_U32 = 4,
  GCAPS_PROBE_LSHRREV_B32 = 5,
  GCAPS_PROBE_MIN_U32 = 6,
  GCAPS_PROBE_TERM = 7,
  GCAPS_PROBE_CNDMASK_SGPR = 8, /* v_cndmask_b32 selecting by a mask held in a scalar register pair */
  GCAPS_PROBE_CMP_CNDMASK = 9,  /* v_cmp_lt_u32 + v_cndmask_b32 (a branch-free minimum): two lane-operations */
  GCAPS_PROBE_KINDS = 10
};
typedef struct {
  int cu_count, clock_khz, wavefront_size, simd_per_cu;
  double spec_lane_ops_per_s;
  double lane_ops_per_s[GCAPS_PROBE_KINDS];
} gcaps_valu_rates;
int gcaps_valu_probe(gcaps_ctx *ctx, gcaps_valu_rates *out);

/*
 * Measured HBM rates of the context's device: what the memory gives plain streaming kernels in practice, the
 * figure beside the published peak in this library's benchmark (no passage of the paper).  For each kind a
 * kernel that reads, writes or copies `bytes` bytes of device memory, 16 bytes per lane and access, is timed
 * alone with events on the context's stream; the call waits for the stream, allocates 2 * bytes of device memory
 * for its duration and frees it.  `_STREAM` kinds give their accesses the non-temporal hint that the analysis
 * kernels give to data they touch once.
 *   bytes            size of each buffer: a multiple of 16, at least 1 MiB; take it well above the 256 MB of the
 *                    memory-side cache (1 GiB in the benchmark)
 *   bytes_per_s[k]   bytes read plus bytes written per second of kind k (a copy moves 2 * bytes)
 * Errors: GCAPS_EINVAL, GCAPS_ENOMEM, GCAPS_EDEVICE.
 */
enum {
  GCAPS_HBM_COPY = 0,
  GCAPS_HBM_COPY_STREAM = 1,
  GCAPS_HBM_READ = 2,
  GCAPS_HBM_READ_STREAM = 3,
  GCAPS_HBM_WRITE = 4,
  GCAPS_HBM_WRITE_STREAM = 5,
  GCAPS_HBM_KINDS = 6
};
typedef struct {
  size_t bytes;
  double bytes_per_s[GCAPS_HBM_KINDS];
} gcaps_hbm_rates;
int gcaps_hbm_probe(gcaps_ctx *ctx, size_t bytes, gcaps_hbm_rates *out);

/* Static description of an error code. */
const char *gcaps_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif
