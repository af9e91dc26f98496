/*
 * fastserve_kvm.h -- C ABI of the proactive key-value cache manager (FastServe,
 * arXiv 2305.05920, Section 4.2) and of the iteration loop that drives the scheduler,
 * the manager and the attention kernels together (Section 3.2 and Algorithm 1).
 *
 * The manager owns the bookkeeping the paper gives its key-value cache manager
 * (Section 3.2): which pool blocks belong to which job, which jobs sit in the pinned
 * host mirror, how many blocks stay idle for new arrivals ("Handling a burst of new
 * jobs"), and which jobs move when, in the order of their estimated next scheduled time
 * ("Job swapping order").  The copies are fs_pool_offload / fs_pool_upload on a side
 * stream of the manager's own, so that the transfer of waiting jobs overlaps the
 * kernels of the running batch ("Overhead-aware swapping": asynchronous memory
 * operations).  Nothing here synchronises the host with the GPU unless a call says so.
 *
 * Blocks are owned by jobs in whole.  A job is resident (all its blocks in HBM),
 * leaving (offload copy in flight), swapped out (all its blocks in host slots) or
 * returning (upload copy in flight).  A model has one pool per layer; the manager takes
 * them all: block ids and host slots are shared by the layers, so one table serves every
 * layer and a job's whole key-value tensor moves together.
 *
 * Block ids and host slots are handed out lowest free id first (a fresh pool hands out
 * 0, 1, 2, ...), so that a job gets neighbouring ids where there are any: neighbouring
 * blocks bound for neighbouring slots travel as one copy.
 *
 * A swap retires, in issue order, once its copy has completed: only then do the blocks an
 * offload vacated (the slots an upload vacated) return to the free lists and does a
 * returning job become schedulable.  Whether a copy has completed is asked of its HIP
 * event without waiting, so a swap may span any number of iterations.
 *
 * All pointers are host pointers unless marked "device".  Every function returns an
 * fs_status (see fastserve.h) unless noted.  Objects are not thread-safe.
 */
#ifndef FASTSERVE_KVM_H
#define FASTSERVE_KVM_H

#include <stdint.h>

#include "fastserve.h"
#include "fastserve_sched.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ===== cache manager (Section 4.2) ================================================== */

typedef struct fs_kvm fs_kvm; /* opaque */

typedef struct fs_kvm_config {
    int32_t num_blocks;          /* HBM blocks per layer pool                               */
    int32_t num_host_blocks;     /* pinned host slots per layer pool                        */
    int32_t block_size;          /* tokens per block (16)                                   */
    int32_t table_width;         /* W: most blocks one job may own; row stride of tables    */
    int32_t reserve_idle_blocks; /* blocks kept idle for new arrivals (fixed part)          */
    int32_t reserve_window;      /* > 0: the reserve also follows the arrival history: the
                                    demands of the last `reserve_window` iterations are kept */
    double reserve_quantile;     /* ... and this quantile of them (0..1) is reserved, never
                                    less than reserve_idle_blocks nor more than half the pool */
    int32_t max_batch;           /* most jobs of one staged batch                           */
    int32_t max_staged_extra;    /* most extra int32 words staged with a batch (>= 0)       */
} fs_kvm_config;

/* layers: the pools of the model's layers (same num_blocks / num_host_blocks / block size as
 * the config), or num_layers == 0 for a manager that keeps the books only and issues no
 * copies (its swaps retire when fs_kvm_retire is told to).  sched: the scheduler whose
 * estimated next scheduled times order the swaps and whose ready flags the manager sets;
 * not owned.  With layers, the pools' GPU must be the current device. */
int fs_kvm_create(const fs_kvm_config *cfg, fs_pool *const *layers, int32_t num_layers, fs_sched *sched,
                  fs_kvm **out);
/* Waits for the manager's copies, then frees everything it allocated. */
int fs_kvm_destroy(fs_kvm *kvm);

/* Blocks that `tokens` tokens occupy; -1 for a NULL manager. */
int32_t fs_kvm_blocks_needed(const fs_kvm *kvm, int64_t tokens);
/* Free HBM blocks / free host slots / current reserve; -1 for a NULL manager. */
int32_t fs_kvm_free_blocks(const fs_kvm *kvm);
int32_t fs_kvm_free_slots(const fs_kvm *kvm);
int32_t fs_kvm_reserve(const fs_kvm *kvm);

/* Once per iteration: the blocks the jobs that arrived in it ask for (0 if none).  Moves
 * the reserve when reserve_window > 0: the ceil(quantile * n)-th smallest of the last n <=
 * window demands (the smallest for quantile 0). */
int fs_kvm_observe_arrivals(fs_kvm *kvm, int32_t blocks_demanded);

/* A new job takes blocks for `tokens` tokens (its prompt and first output) and is resident,
 * length 0.  FS_ERR_OOM, and no change, if fewer blocks are free or the job would need more
 * than table_width blocks; FS_ERR_INVALID_ARG for an id already present. */
int fs_kvm_admit(fs_kvm *kvm, int64_t job_id, int64_t tokens);
/* Room for `new_tokens` more tokens of a resident job: *ok = 1 and the blocks are taken, or
 * *ok = 0 and nothing changes (HBM full or table_width reached). */
int fs_kvm_grow(fs_kvm *kvm, int64_t job_id, int32_t new_tokens, int32_t *ok);
/* The job's cache now holds `tokens` more tokens. */
int fs_kvm_advance(fs_kvm *kvm, int64_t job_id, int32_t tokens);
/* The job leaves.  Its blocks and slots return to the free lists at once, except those a
 * copy in flight still reads or writes: they return when that swap retires. */
int fs_kvm_release(fs_kvm *kvm, int64_t job_id);

/* Issues this iteration's swaps on the side stream, which first waits (on the GPU) for
 * everything `compute_stream` (a hipStream_t, device work queue of the decode kernels) has
 * been given so far.  With margin = reserve + want_free:
 *   out: resident jobs that are not in `running` leave, largest estimated next scheduled
 *        time first, until free blocks plus the blocks of offloads in flight reach the
 *        margin; a job that does not fit the free host slots is passed over;
 *   in:  swapped-out jobs return, smallest estimated next scheduled time first, as long as
 *        the free blocks left after taking theirs stay at or above the margin.
 * A job that leaves is marked not ready in the scheduler at once; a job that returns
 * becomes ready when its swap retires. */
int fs_kvm_start_swaps(fs_kvm *kvm, const int64_t *running, int32_t n_running, int32_t want_free,
                       void *compute_stream);
/* Retires completed swaps, oldest first, at most max_swaps of them (< 0: no limit).
 * wait != 0 waits on the host for each copy instead of stopping at the first one still in
 * flight.  A manager without layers has no copies: every swap counts as completed.
 * *retired (optional) receives the number retired. */
int fs_kvm_retire(fs_kvm *kvm, int32_t max_swaps, int32_t wait, int32_t *retired);

/* State of one job; any output pointer may be NULL.  state: 0 resident, 1 leaving,
 * 2 swapped out, 3 returning.  ids receives min(cap, n) block ids (states 0, 3) or host
 * slots (states 1, 2) in logical order, *n their full number. */
int fs_kvm_job_info(const fs_kvm *kvm, int64_t job_id, int32_t *state, int64_t *length, int32_t *ids,
                    int32_t cap, int32_t *n);
/* Totals since creation, counted per layer pool (blocks moved x layers). */
int fs_kvm_stats(const fs_kvm *kvm, int64_t *blocks_out, int64_t *blocks_in, int32_t *swaps_in_flight);

/* Block-table rows of `n` resident jobs, table_width entries each, unused entries -1
 * (host array, n * table_width int32). */
int fs_kvm_table_rows(const fs_kvm *kvm, const int64_t *job_ids, int32_t n, int32_t *rows);

/* The device-side inputs of one batch: table rows, lengths (tokens cached) and n_extra
 * caller words (e.g. prompt token offsets) of the n jobs are written into a pinned staging
 * slot and brought to the GPU by a small copy kernel launched on `stream`, the stream the
 * kernels will run on (every call on one manager names the same stream): the words are in
 * place, in stream order, before anything launched on it afterwards.
 * *d_table, *d_lens, *d_extra receive device pointers that stay valid until 47 later
 * batches have been staged.  Needs layers; n <= max_batch, n_extra <= max_staged_extra. */
int fs_kvm_stage_batch(fs_kvm *kvm, const int64_t *job_ids, int32_t n, const int32_t *extra, int32_t n_extra,
                       void *stream, const int32_t **d_table, const int32_t **d_lens, const int32_t **d_extra);

/* ===== iteration loop (Section 3.2, Algorithm 1) ==================================== */

typedef struct fs_serve fs_serve; /* opaque: owns a scheduler and a cache manager */

typedef struct fs_serve_config {
    int32_t num_queues;  /* scheduler: see fs_sched_create                                  */
    double q1;
    int32_t eta;
    double alpha;
    int32_t max_batch;
    int64_t max_prompt_tokens; /* most prompt tokens one iteration may pack (0 = no limit): a
                                  first-iteration job that would exceed it waits for the next */
    fs_kvm_config kvm;   /* max_batch and max_staged_extra are set by the loop              */
} fs_serve_config;

/* Device buffers the kernels of an iteration read and write (pool dtype; all rows of a
 * layer's call are taken from the front of the buffers).  prompt_*: [max_prompt_tokens][H][D],
 * decode_*: [max_batch][H][D]; the outputs float32.  The same buffers serve every layer. */
typedef struct fs_serve_buffers {
    const void *prompt_q, *prompt_k, *prompt_v; /* device */
    float *prompt_out;                          /* device */
    int64_t max_prompt_tokens;
    const void *decode_q, *decode_k, *decode_v; /* device */
    float *decode_out;                          /* device */
} fs_serve_buffers;

/* What fs_serve_plan decided for the coming iteration (host arrays owned by the loop,
 * valid until the next fs_serve_plan). */
typedef struct fs_serve_iteration {
    int64_t iteration;
    int32_t n_first;              /* jobs running their initialization phase              */
    const int64_t *first_ids;
    const int32_t *token_offsets; /* n_first + 1 offsets of their prompts, packed         */
    int64_t prompt_tokens;
    int32_t n_decode;             /* jobs running a decoding step                         */
    const int64_t *decode_ids;
    const int32_t *lens_before;   /* tokens each of them has cached                       */
    int32_t n_waiting;            /* submitted jobs not yet admitted                      */
    int32_t n_unfinished;         /* jobs submitted and not finished (0: nothing left)    */
} fs_serve_iteration;

typedef struct fs_serve_stats {
    int64_t iterations, job_tokens, prompt_tokens, finished_jobs;
    int64_t blocks_swapped_out, blocks_swapped_in;
    int64_t iterations_without_work;
    /* host time fs_serve_run spent in the three calls of its iterations (seconds) */
    double host_seconds_plan, host_seconds_launch, host_seconds_complete;
} fs_serve_stats;

int fs_serve_create(const fs_serve_config *cfg, fs_pool *const *layers, int32_t num_layers, fs_serve **out);
int fs_serve_destroy(fs_serve *s);
fs_sched *fs_serve_scheduler(fs_serve *s); /* NULL for a NULL loop */
fs_kvm *fs_serve_manager(fs_serve *s);

/* A job that arrives at iteration `arrival_iteration` (>= the current one) with
 * `prompt_tokens` >= 1 input tokens and `output_tokens` >= 1 tokens to generate (the first
 * of them by the initialization phase).  init_time / decode_time: its profiled iteration
 * times (Section 3.2, job profiler) for the scheduler. */
int fs_serve_submit(fs_serve *s, int64_t job_id, int64_t arrival_iteration, int32_t prompt_tokens,
                    int32_t output_tokens, double init_time, double decode_time);

/* One iteration in three calls (the caller may fill the buffers between plan and launch):
 *   plan:     arrivals of this iteration join the waiting list; waiting jobs are admitted,
 *             oldest first, while their blocks fit beside the reserve; completed swaps
 *             retire; the scheduler picks the batch; decoding jobs take room for one more
 *             token (one that finds none sits the iteration out); swaps are started.
 *   launch:   fs_prefill_step over the first-iteration jobs and fs_decode_step over the
 *             decoding jobs of layer `layer` (-1: every layer in turn, from the same
 *             buffers), on `stream`; tables and lengths reach the GPU through
 *             fs_kvm_stage_batch, once per iteration.  A model calls it once per layer,
 *             with that layer's projections in the buffers.  Needs layers.
 *   complete: lengths advance, every job that ran has produced one token, jobs that have
 *             produced all theirs leave, the scheduler is told (elapsed = the largest
 *             profiled time among the jobs that ran, q1 if none ran). */
int fs_serve_plan(fs_serve *s, void *stream, fs_serve_iteration *it);
int fs_serve_launch(fs_serve *s, int32_t layer, const fs_serve_buffers *buf, void *stream);
int fs_serve_complete(fs_serve *s);

/* plan + launch + complete until every submitted job has finished or max_iterations
 * iterations have run; the host never waits for the GPU inside the loop (the caller
 * synchronises `stream` afterwards). */
int fs_serve_run(fs_serve *s, const fs_serve_buffers *buf, void *stream, int64_t max_iterations,
                 fs_serve_stats *stats);
int fs_serve_get_stats(const fs_serve *s, fs_serve_stats *stats);

#ifdef __cplusplus
}
#endif
#endif /* FASTSERVE_KVM_H */
