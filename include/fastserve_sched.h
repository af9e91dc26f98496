/*
 * fastserve_sched.h -- C ABI of the host-side serving policy that feeds the decode
 * step: the skip-join multi-level feedback queue scheduler (FastServe, arXiv
 * 2305.05920, Section 4.1 and Algorithm 1) and the swap-order estimate of the
 * proactive key-value cache manager (Section 4.2, "Job swapping order").
 *
 * All pointers are host pointers.  Every function returns an fs_status (see
 * fastserve.h) unless noted.  A scheduler object is not thread-safe.
 *
 * Model (one call pair per iteration):
 *   ids  = fs_sched_schedule(...)              pick at most max_batch ready jobs
 *   ... run one iteration on them (fs_decode_step) ...
 *   fs_sched_complete_iteration(ids, elapsed, finished)
 * Queues Q_1..Q_n (1 = highest priority) have quanta q_k = q1 * 2^(k-1).
 *   - A new job joins the highest-priority queue whose quantum covers its first
 *     (initialization) iteration time: min i such that q_i >= init_time, else Q_n.
 *   - Every job that ran is charged the iteration's elapsed time; when its use
 *     reaches its queue's quantum it moves eta queues down (further if its next
 *     iteration would not fit that quantum), to the back, with a fresh quantum.
 *   - Every job that did not run accumulates waiting time; at alpha or more it moves
 *     to the back of Q_1 with a fresh quantum and its waiting time restarts.
 *   - Jobs are visited in queue order (Q_1 first, first-in first-out inside a queue).
 *   - A job marked not ready (its key-value blocks are not in GPU memory) keeps its
 *     place but is passed over by fs_sched_schedule.
 */
#ifndef FASTSERVE_SCHED_H
#define FASTSERVE_SCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fs_sched fs_sched; /* opaque */

/* num_queues >= 1, q1 > 0 (quantum of Q_1 = the minimum iteration time), eta >= 1,
 * alpha > 0 (starvation threshold, same unit as the times), max_batch >= 1. */
int fs_sched_create(int32_t num_queues, double q1, int32_t eta, double alpha, int32_t max_batch,
                    fs_sched **out);
int fs_sched_destroy(fs_sched *s);

/* Skip-join of a new job (Algorithm 1, lines 6-9).  init_time: profiled time of its
 * first iteration; decode_time: of each later one.  *queue_out (optional) receives the
 * queue it joined.  A job id already present -> FS_ERR_INVALID_ARG. */
int fs_sched_add_job(fs_sched *s, int64_t job_id, double init_time, double decode_time,
                     int32_t *queue_out);

/* Residency of the job's key-value blocks (isReady of Algorithm 1). */
int fs_sched_set_ready(fs_sched *s, int64_t job_id, int32_t ready);

/* Algorithm 1, lines 23-27: up to min(cap, max_batch) ready jobs in priority order. */
int fs_sched_schedule(const fs_sched *s, int64_t *out_ids, int32_t cap, int32_t *n_out);

/* Algorithm 1, lines 11-22, after an iteration of `elapsed` time units that ran the
 * jobs `ran`; `finished` (a subset of ran) leave the system. */
int fs_sched_complete_iteration(fs_sched *s, const int64_t *ran, int32_t n_ran, double elapsed,
                                const int64_t *finished, int32_t n_finished);

/* State of one job; any output pointer may be NULL. */
int fs_sched_job_info(const fs_sched *s, int64_t job_id, int32_t *priority, double *used,
                      double *starve, int64_t *iterations);
int32_t fs_sched_num_jobs(const fs_sched *s); /* -1 for a NULL scheduler */

/* Section 4.2: T_promote(i) = alpha - waited(i) (not below 0);
 * T_execute(i) = (1/B) * sum over jobs j in higher-priority queues of the quanta of the
 * queues j is demoted through down to job i's queue (q_{p_j} + ... + q_{p_i - 1});
 * ENST(i) = min of the two.  Any output pointer may be NULL. */
int fs_sched_enst(const fs_sched *s, int64_t job_id, double *t_promote, double *t_execute, double *enst);

/* Orders n candidate job ids for swapping: swap_in = 0 -> largest ENST first (swap out
 * order), swap_in != 0 -> smallest ENST first.  Ties: the job in the lower-priority queue
 * leaves first / the higher-priority one returns first, then by id.  `ordered` receives
 * the n ids. */
int fs_sched_swap_order(const fs_sched *s, const int64_t *candidates, int32_t n, int32_t swap_in,
                        int64_t *ordered);

#ifdef __cplusplus
}
#endif
#endif /* FASTSERVE_SCHED_H */
