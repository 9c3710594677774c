/*
 * CPU oracle for the GCAPS response-time analyses.  TEST INFRASTRUCTURE ONLY.
 *
 * This is the slow, plain, single-threaded reference that the tests, the smoke
 * check and the benchmark's CPU-baseline leg compare the GPU library against.
 * The product library never includes, links or calls anything in this
 * directory, and nothing here includes anything of the product library.
 *
 * What it computes: for one taskset of the task model of Sec. 3 (sporadic,
 * fixed-priority, constrained-deadline tasks partitioned onto CPU cores, each
 * a sequence of CPU segments and GPU segments G_{i,j} = (G^m_{i,j}, G^e_{i,j})),
 * the worst-case response-time bound R_i = C_i + G_i + I^C_i + I^G_i (Eq. 1,
 * 2, 4) of every task under one of four analyses:
 *   - default round-robin TSG scheduling, busy-waiting   (Lemmas 1-5)
 *   - default round-robin TSG scheduling, self-suspension (Lemmas 1-3, 6, 7)
 *   - GCAPS preemptive priority scheduling, busy-waiting  (Lemmas 8-12)
 *   - GCAPS preemptive priority scheduling, self-suspension (Lemmas 8, 9, 13-15)
 * R_i appears on both sides of each bound, so it is obtained as the least
 * fixed point of the recurrence, iterated from the R-independent part.
 *
 * All times are integer microseconds.  Results are int64.
 *
 * Pins: every analysis is pinned by tests that do not go through this code
 * (hand-worked fixed points, the classic uniprocessor RTA special case, the
 * pass/fail verdict the paper prints for the taskset of Table 2, an
 * exhaustive least-fixed-point search, monotonicity, and a discrete-event
 * simulation that must never exceed the bound).  Table 5's WCRT column is NOT
 * a pin (its inputs are not printed): parity unpinned for that table.
 */
#ifndef GCAPS_RTA_ORACLE_H
#define GCAPS_RTA_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* analysis selectors */
#define ORACLE_POLICY_GCAPS 1 /* Sec. 5.3 */
#define ORACLE_POLICY_RR 2    /* Sec. 5.2 */
#define ORACLE_WAIT_BUSY 0
#define ORACLE_WAIT_SUSPEND 1

/* option bits */
#define ORACLE_OPT_LITERAL_LEMMA10 1u /* keep the eta^g_i > 0 guard on the same-core sum of Lemma 10 */
/* Go on after a task whose bound exceeds its deadline: its response time is unknown, so the
 * jitters J^c_h, J^g_h of the tasks below it take D_h in place of R_h (proof of Lemma 10).  Every
 * task is analysed: resp[i] = R_i or ORACLE_RESP_MISS, never ORACLE_RESP_NOT_ANALYSED; the verdict
 * is unchanged.  Pins: equal to the default up to the first miss, a hand-worked four-task example,
 * bounds never above those with D_h in every jitter (Sec. 5.4 with GPU = CPU priorities). */
#define ORACLE_OPT_CONTINUE_AFTER_MISS 2u

/* response-time sentinels */
#define ORACLE_RESP_MISS (-1)         /* first task (in priority order) whose bound exceeds D_i */
#define ORACLE_RESP_NOT_ANALYSED (-2) /* every lower-priority task after a miss */

/* error codes */
#define ORACLE_OK 0
#define ORACLE_EINVAL (-1) /* null pointer, zero sizes, unknown selector */
#define ORACLE_ETASK (-2)  /* a task or parameter violates the task model */
#define ORACLE_EORDER (-3) /* GPU priorities that disagree with the CPU priorities on one core (Sec. 4.3) */

/*
 * One taskset.  Arrays are in caller order, any priority order.
 *   n_tasks   n            (1..255)
 *   max_gseg  S: slots per task in gm_us/ge_us (0..255); slots >= n_gseg[i] are ignored
 *   theta_us  GPU context-switch overhead theta (Def. 1)
 *   eps_us    runlist-update delay epsilon = alpha + theta (Def. 2)
 *   slice_us  TSG time slice L >= 1 (Eq. 3)
 *   cpu_us[i]      C_i    period_us[i]  T_i >= 1    deadline_us[i]  1 <= D_i <= T_i
 *   prio[i]        larger = higher; ties broken by lower caller index first
 *   core[i]        CPU core of tau_i
 *   n_gseg[i]      eta^g_i <= S
 *   gm_us[i*S+j], ge_us[i*S+j]   G^m_{i,j}, G^e_{i,j}
 * Outputs (caller order): resp[i] = R_i, or a sentinel; *sched = 1 iff no task missed.
 * *terms (may be NULL) receives the number of ceil(.)*cost terms evaluated.
 */
int oracle_rta_taskset(uint32_t n_tasks, uint32_t max_gseg, uint32_t theta_us, uint32_t eps_us,
                       uint32_t slice_us, const uint32_t *cpu_us, const uint32_t *period_us,
                       const uint32_t *deadline_us, const int32_t *prio, const uint8_t *core,
                       const uint8_t *n_gseg, const uint32_t *gm_us, const uint32_t *ge_us,
                       int policy, int wait_mode, uint32_t options, int64_t *resp, uint8_t *sched,
                       uint64_t *terms);

/*
 * A batch of n_tasksets tasksets with the same n_tasks and max_gseg; per-taskset
 * parameter arrays [n_tasksets], per-task arrays [n_tasksets*n_tasks], per-segment
 * arrays [n_tasksets*n_tasks*max_gseg].  policy_mask is a bit-or of the policy
 * selectors; outputs are resp[p][taskset][task] and sched[p][taskset] with p
 * running over the selected policies in increasing selector value.
 * threads = 1 runs everything in the calling thread; threads > 1 hands disjoint
 * ranges of tasksets to that many std::thread workers, each running the same
 * single-threaded routine.  *first_bad (may be NULL) gets the index of the first
 * invalid taskset when ORACLE_ETASK is returned.
 */
int oracle_rta_batch(uint32_t n_tasksets, uint32_t n_tasks, uint32_t max_gseg,
                     const uint32_t *theta_us, const uint32_t *eps_us, const uint32_t *slice_us,
                     const uint32_t *cpu_us, const uint32_t *period_us, const uint32_t *deadline_us,
                     const int32_t *prio, const uint8_t *core, const uint8_t *n_gseg,
                     const uint32_t *gm_us, const uint32_t *ge_us, int policy_mask, int wait_mode,
                     uint32_t options, int threads, int64_t *resp, uint8_t *sched,
                     uint64_t *terms_total, uint32_t *first_bad);

/*
 * Sec. 5.4: the GCAPS analysis of one taskset when the GPU segments of tau_i run at a
 * priority gprio[i] of their own (larger = higher; equal values fall back to the CPU priority
 * order).  Against oracle_rta_taskset with ORACLE_POLICY_GCAPS:
 *   - the sums over higher-priority tasks of OTHER cores (second sums of Lemmas 10 and 13,
 *     Lemma 11) run over the tasks with a higher GPU priority; hpp(tau_i) is unchanged;
 *   - every release jitter is taken with D_h in place of R_h.
 * The bounds of different tasks then do not depend on each other: every task is analysed,
 * resp[i] = R_i or ORACLE_RESP_MISS, *sched = 1 iff none missed.  theta and L play no part.
 * Returns ORACLE_EORDER when two tasks of one core are ordered differently by prio and gprio.
 */
int oracle_gprio_rta_taskset(uint32_t n_tasks, uint32_t max_gseg, uint32_t eps_us,
                             const uint32_t *cpu_us, const uint32_t *period_us,
                             const uint32_t *deadline_us, const int32_t *prio, const uint8_t *core,
                             const uint8_t *n_gseg, const uint32_t *gm_us, const uint32_t *ge_us,
                             const int32_t *gprio, int wait_mode, uint32_t options, int64_t *resp,
                             uint8_t *sched, uint64_t *terms);

/* The same for every taskset of a batch (gprio and resp [n_tasksets*n_tasks], sched [n_tasksets]);
 * stops at the first taskset that is invalid or whose priorities disagree on a core (*first_bad). */
int oracle_gprio_rta_batch(uint32_t n_tasksets, uint32_t n_tasks, uint32_t max_gseg, const uint32_t *eps_us,
                           const uint32_t *cpu_us, const uint32_t *period_us, const uint32_t *deadline_us,
                           const int32_t *prio, const uint8_t *core, const uint8_t *n_gseg,
                           const uint32_t *gm_us, const uint32_t *ge_us, const int32_t *gprio, int wait_mode,
                           uint32_t options, int64_t *resp, uint8_t *sched, uint32_t *first_bad);

/*
 * Sec. 4.3: search for GPU-segment priorities by Audsley's scheme.  Levels are handed out
 * from the lowest (1) to the highest (n).  At each level the unassigned tasks are tried from
 * the lowest to the highest CPU priority; a task is a candidate only if no unassigned task of
 * its core has a lower CPU priority (the two orders must agree on a core); the first candidate
 * whose bound of Sec. 5.4 - with every other unassigned task above it - meets its deadline
 * takes the level.  The search fails when a level finds no task, or (checked first) when some
 * task's own demand C_i + G_i + 2*eps*eta_i + (eta_i + 1)*eps exceeds D_i.
 * Outputs (caller order): success: gprio[i] = level of tau_i, resp[i] = its bound at that
 * level, *sched = 1; failure: gprio[i] = 0, resp[i] = ORACLE_RESP_NOT_ANALYSED, *sched = 0.
 *
 * Pins: the taskset of Table 2 (printed: fails with GPU = CPU priorities, passes with tau_4
 * above tau_3; hand-worked bounds), agreement with oracle_rta_taskset where Sec. 5.4 changes
 * nothing, an exhaustive search over all admissible priority orders of small tasksets
 * (Audsley's scheme finds an order iff one exists), and the discrete-event simulator run
 * with the assigned GPU priorities.
 */
int oracle_gprio_assign_taskset(uint32_t n_tasks, uint32_t max_gseg, uint32_t eps_us,
                                const uint32_t *cpu_us, const uint32_t *period_us,
                                const uint32_t *deadline_us, const int32_t *prio, const uint8_t *core,
                                const uint8_t *n_gseg, const uint32_t *gm_us, const uint32_t *ge_us,
                                int wait_mode, uint32_t options, int32_t *gprio, int64_t *resp,
                                uint8_t *sched, uint64_t *terms);

/*
 * The search for every taskset of a batch (layout as oracle_rta_batch; gprio and resp are
 * [n_tasksets*n_tasks], sched [n_tasksets]).  skip (may be NULL): tasksets with skip[s] != 0
 * are not searched (they passed the test with GPU = CPU priorities): gprio = 0, resp =
 * ORACLE_RESP_NOT_ANALYSED, sched = 1.
 */
int oracle_gprio_assign_batch(uint32_t n_tasksets, uint32_t n_tasks, uint32_t max_gseg,
                              const uint32_t *eps_us, const uint32_t *cpu_us, const uint32_t *period_us,
                              const uint32_t *deadline_us, const int32_t *prio, const uint8_t *core,
                              const uint8_t *n_gseg, const uint32_t *gm_us, const uint32_t *ge_us,
                              const uint8_t *skip, int wait_mode, uint32_t options, int threads,
                              int32_t *gprio, int64_t *resp, uint8_t *sched, uint64_t *terms_total,
                              uint32_t *first_bad);

#ifdef __cplusplus
}
#endif
#endif
