/*
 * fastserve.h -- C ABI of the paged attention iterations for AMD MI355X (gfx950).
 *
 * One iteration of token-granularity preemptive serving (FastServe,
 * arXiv 2305.05920): the scheduler admits a ragged batch of jobs (Section 3.2,
 * Algorithm 1).  In the decoding phase the engine appends every job's new
 * key/value token to that job's cache and runs the new token's masked
 * self-attention over the whole cache; in the initialization phase (a job's
 * first iteration) it fills the cache with all prompt tokens and runs their
 * causal self-attention (Section 2.2).  The cache manager moves blocks of
 * inactive jobs between GPU memory and host memory (Section 4.2).
 *
 * Conventions
 *   - Every function returns an fs_status (0 = FS_OK, negative = error) unless
 *     noted.  No exception crosses this boundary.
 *   - "device pointer" = HBM address valid on the pool's GPU; "host pointer" =
 *     ordinary process memory.  The library never takes ownership of a pointer
 *     it is given; the caller keeps q/k/v/out/tables/lengths alive until the
 *     stream has run the call.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     that take a stream are asynchronous on it.
 *   - A pool is not thread-safe; different pools may be used concurrently.
 *     The pool's GPU must be the current device of the calling thread.
 *   - The library never allocates or frees block ids: which block holds which
 *     tokens is decided by the caller (the paper's key-value cache manager,
 *     Section 3.2) and handed over as a block table.
 *
 * Pool layout (this library's choice; the paper fixes only block-grained
 * allocation, Section 2.2).  With e = bytes per element, x = 16/e elements per
 * 16-byte vector, B = block_size tokens, H = num_heads, D = head_dim, block b
 * starts at byte b * fs_pool_block_bytes() and holds 2*H*B*D elements, the K
 * region followed by the V region:
 *     K[h][slot][d]  at element ((h*(D/x) + d/x)*B + slot)*x + d%x
 *     V[h][slot][d]  at element H*B*D + (h*B + slot)*D + d
 * so each (block, head) chunk of K or of V is B*D*e contiguous bytes (4 KiB at
 * B=16, D=128, bf16), and one block is one contiguous copy for offload/upload.
 * Logical token t of a job lives in block block_table[job][t / B], slot t % B.
 */
#ifndef FASTSERVE_H
#define FASTSERVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fs_pool fs_pool; /* opaque; created and destroyed by the library */

typedef enum fs_dtype {
    FS_BF16 = 0, /* 2-byte bfloat16 pool, q, k, v                         */
    FS_F32 = 1,  /* 4-byte IEEE float pool, q, k, v                       */
    FS_F16 = 2   /* 2-byte IEEE half pool, q, k, v (the precision of the
                    paper's runs, Section 6.1)                            */
} fs_dtype;

typedef enum fs_status {
    FS_OK = 0,
    FS_ERR_INVALID_ARG = -1, /* null pointer, negative count, size out of range       */
    FS_ERR_OOM = -2,         /* device or pinned-host allocation failed               */
    FS_ERR_BAD_TABLE = -3,   /* a kernel met a block id or length outside the pool    */
    FS_ERR_HIP = -4,         /* a HIP runtime call failed                              */
    FS_ERR_UNSUPPORTED = -5  /* dtype / head_dim / block_size combination not built   */
} fs_status;

typedef struct fs_pool_config {
    int32_t dtype;           /* fs_dtype of pool, q, k, v                               */
    int32_t num_heads;       /* heads resident on this GPU (key/value heads == query
                                heads: the paper's models are multi-head, Table 1)     */
    int32_t head_dim;        /* 64 or 128                                               */
    int32_t block_size;      /* tokens per block; 16                                    */
    int32_t num_blocks;      /* HBM blocks in the pool                                  */
    int32_t num_host_blocks; /* pinned-host slots for offload; 0 = none                 */
    int32_t max_jobs;        /* hint: largest num_jobs of one call (sizes scratch);
                                0 = 1024.  Larger batches still work: they run in
                                slices of this many jobs.                                */
    int32_t max_workgroups;  /* cap on the attention grid in workgroups; 0 = none       */
    float scale;             /* softmax scale; 0 = 1/sqrt(head_dim)                     */
    int32_t reserved;        /* must be 0                                               */
    void *device_mem;        /* optional caller-owned HBM for the blocks (device
                                pointer, 256-byte aligned); NULL = library allocates   */
    size_t device_bytes;     /* size of device_mem; >= num_blocks * block bytes         */
} fs_pool_config;

/* ---- pool (Section 2.2 block-grained cache; Section 4.2 host extension) ---------- */

/* Creates the block pool on the current device, its scratch buffers and, if
 * num_host_blocks > 0, a pinned host mirror of that many block slots.
 * Block contents start undefined.  *out is written only on FS_OK. */
int fs_pool_create(const fs_pool_config *cfg, fs_pool **out);

/* Synchronises the device and frees everything the library allocated. */
int fs_pool_destroy(fs_pool *pool);

/* Bytes of one block = 2*H*B*D*e.  Returns 0 for a NULL pool. */
size_t fs_pool_block_bytes(const fs_pool *pool);

/* Device pointer to block 0 (the caller's device_mem if one was given). */
void *fs_pool_device_ptr(const fs_pool *pool);

/* Synchronous copy of one whole block between host memory and the pool
 * (test and harness helper; host pointer, fs_pool_block_bytes() bytes). */
int fs_pool_write_block(fs_pool *pool, int32_t block_id, const void *host_src);
int fs_pool_read_block(const fs_pool *pool, int32_t block_id, void *host_dst);

/* Kernels never dereference a block id outside [0, num_blocks) or a position
 * beyond table_stride*B: they skip it and raise a flag in device memory.
 * fs_pool_check waits for `stream`, returns FS_ERR_BAD_TABLE if the flag was
 * raised since the last check, and clears it. */
int fs_pool_check(fs_pool *pool, void *stream);

/* ---- KV append (Section 2.2, decoding phase: the new token's key and value join
 *      the cache) ------------------------------------------------------------------
 * For every job j: copies k[j], v[j] (device, [num_jobs][H][D], pool dtype) to
 * logical position p = job_lens[j], i.e. block block_table[j*table_stride + p/B],
 * slot p%B.  A bit copy: no conversion.
 *   block_table: device int32 [num_jobs][table_stride]; entries beyond a job's
 *                blocks are ignored.  The entry for p/B must already name a block
 *                the caller allocated.
 *   job_lens:    device int32 [num_jobs], tokens already cached (the write position).
 * Two jobs must not append into the same (block, slot). */
int fs_kv_append(fs_pool *pool, const int32_t *block_table, int32_t table_stride,
                 const int32_t *job_lens, int32_t num_jobs, const void *k, const void *v,
                 void *stream);

/* ---- bulk KV write (Section 2.2, initialization phase: the first iteration builds
 *      the cache of all prompt tokens) -----------------------------------------------
 * Job j receives tokens [token_offsets[j], token_offsets[j+1]) of the packed
 * arrays k, v (device, [total_tokens][H][D], pool dtype) at logical positions
 * job_starts[j], job_starts[j]+1, ...
 *   job_starts:    device int32 [num_jobs]
 *   token_offsets: device int32 [num_jobs+1], non-decreasing, [0] = 0,
 *                  [num_jobs] = total_tokens
 *   total_tokens:  the same total, known to the host (sizes the launch). */
int fs_kv_prefill(fs_pool *pool, const int32_t *block_table, int32_t table_stride,
                  const int32_t *job_starts, const int32_t *token_offsets, int32_t num_jobs,
                  int64_t total_tokens, const void *k, const void *v, void *stream);

/* ---- prompt attention (Section 2.2 and Figure 3, initialization phase: the first
 *      iteration of a job processes all its input tokens; masked self-attention lets
 *      token i see tokens 0..i of its own prompt) -----------------------------------
 * For every job j and every token i of its prompt:
 *     out[t0+i][h][:] = sum_{t<=i} softmax_t(scale * q[t0+i][h] . k[t0+t][h]) * v[t0+t][h][:]
 * with t0 = token_offsets[j].  The keys and values are read from the packed projection
 * arrays (the same ones fs_kv_prefill writes into the pool), not from the pool; the pool
 * handle supplies dtype, H, D and scale.  Runs on the matrix cores with fp32
 * accumulation; the softmax weights are rounded to the pool dtype before they multiply
 * the values.
 *   q, k, v:       device [total_tokens][H][D], pool dtype (FS_BF16 or FS_F16;
 *                  FS_F32 pools return FS_ERR_UNSUPPORTED)
 *   token_offsets: device int32 [num_jobs+1], non-decreasing, [0] = 0,
 *                  [num_jobs] = total_tokens
 *   total_tokens:  the same total, known to the host.  A job whose offsets decrease or
 *                  leave [0, total_tokens] raises the pool's error flag (fs_pool_check)
 *                  and its rows are not written; so does a launch with more than 262144
 *                  work items (128 query rows x 8 heads each), which is served in part.
 *   out:           device float32 [total_tokens][H][D]; every row of a valid job is
 *                  written.
 * A one-workgroup kernel first derives the work list from the offsets on the device
 * (longest jobs and largest query tiles first); the host needs no prompt length.
 * Asynchronous on `stream`; nothing is allocated; calls on one pool share the list and
 * must be ordered by the stream. */
int fs_prefill_attention(fs_pool *pool, const void *q, const void *k, const void *v,
                         const int32_t *token_offsets, int32_t num_jobs, int64_t total_tokens,
                         float *out, void *stream);

/* ---- whole initialization phase of a batch of new jobs in one launch (Section 2.2:
 *      the first iteration builds the cache of all prompt tokens and computes their
 *      attention; Sections 5-6 on fusing operations into fewer kernels) ---------------
 * fs_prefill_attention plus the cache fill of fs_kv_prefill with job_starts = 0: token t
 * of job j is also written to slot t % block_size of block block_table[j][t / block_size]
 * (bit copy), by the workgroup that has the token's key/value tile staged.  Arguments as
 * in those two calls; a table entry outside [0, num_blocks) or a prompt longer than
 * table_stride blocks raises the error flag and that write is skipped.
 * Jobs must own disjoint blocks. */
int fs_prefill_step(fs_pool *pool, const int32_t *block_table, int32_t table_stride,
                    const int32_t *token_offsets, int32_t num_jobs, int64_t total_tokens,
                    const void *k, const void *v, const void *q, float *out, void *stream);

/* ---- decode attention (Section 2.2: masked self-attention of the one new token
 *      over the keys and values of all tokens up to and including itself) ------------
 * For every job j and head h, with L = job_lens[j] (tokens to attend over, i.e.
 * the length after this step's append):
 *     s_t = scale * <q[j][h], K_j[t][h]>,  w = softmax_t(s),  out[j][h] = sum_t w_t V_j[t][h]
 *   q:   device [num_jobs][H][D], pool dtype
 *   out: device float32 [num_jobs][H][D]; rows of a job with L == 0 are set to 0
 *   max_len_hint: an upper bound of max_j job_lens[j] known to the host (sizes the
 *                launch only; <= 0 means table_stride*B).  Lengths are read on the
 *                device; the host is never synchronised.
 * Uses the pool's scratch: two calls on one pool must not overlap in time. */
int fs_decode_attention(const void *q, fs_pool *pool, const int32_t *block_table,
                        int32_t table_stride, const int32_t *job_lens, int32_t num_jobs,
                        int32_t max_len_hint, float *out, void *stream);

/* ---- decode attention for callers that cannot allocate ------------------------------
 * For callers that must not reach an allocating call: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same operation, arguments and result
 * (bit for bit) as fs_decode_attention, but the partial results and the step plan live in
 * a fixed device array that is part of the library image (1 069 312 bytes per GPU, held
 * until the process ends) instead of the pool's allocated scratch, the launches are plain
 * ones even while fs_profile_enable is on (no events are created), and the
 * "merge_in_kernel" knob is ignored (the two-launch form always).  The call allocates and
 * frees nothing.
 *   Limits: num_jobs <= 1024 in one call (larger batches are refused with
 *   FS_ERR_INVALID_ARG, not sliced); head_dim <= 128; the attention grid is at most 256
 *   workgroups.
 *   Every call on one GPU shares that GPU's array, whichever pool it names: calls that
 *   overlap in time on one GPU race, also across pools and streams.  The array keeps the
 *   last call's contents; the kernels write every cell they later read, so nothing needs
 *   clearing between calls. */
int fs_decode_attention_static(const void *q, fs_pool *pool, const int32_t *block_table,
                               int32_t table_stride, const int32_t *job_lens, int32_t num_jobs,
                               int32_t max_len_hint, float *out, void *stream);

/* ---- fused decode step (Sections 2.2 and 5: one iteration appends and attends; the
 *      paper's engine fuses operations into fewer kernels) ---------------------------
 * Same result as fs_kv_append(pool, table, stride, job_lens, J, k, v) followed by
 * fs_decode_attention over job_lens[j] + 1 tokens, in one kernel launch fewer: the
 * attention kernel takes the new token's key and value from k, v instead of the pool, and
 * the rows are written into the pool by the launch that merges the partial results (or by
 * the attention kernel itself, see "append_in_attention").
 *   job_lens: device int32 [num_jobs], tokens cached BEFORE this step (as for append)
 *   k, v, q:  device [num_jobs][H][D], pool dtype;  out: device float32 [num_jobs][H][D]
 *   max_len_hint: upper bound of max_j job_lens[j] + 1 (<= 0: table_stride*B)
 * Sums run in a different order than in the two-call form, so outputs agree with it
 * to rounding, not bit for bit; the pool contents afterwards are identical. */
int fs_decode_step(fs_pool *pool, const int32_t *block_table, int32_t table_stride,
                   const int32_t *job_lens, int32_t num_jobs, const void *k, const void *v,
                   const void *q, int32_t max_len_hint, float *out, void *stream);

/* ---- block offload / upload (Section 4.2: key-value tensors of inactive jobs are
 *      swapped out to host memory and swapped in before the job is scheduled) --------
 * Copies n whole blocks between pool blocks block_ids[i] and pinned host slots
 * host_slots[i] (host int32 arrays, read before return), asynchronously on
 * `stream`.  Upload may target any block id; the caller patches its tables.
 * By default each run of consecutive (block id, host slot) pairs is one
 * hipMemcpyAsync on the copy engines, which leaves the compute units to a decode
 * step running on another stream; knob "swap_engine" = 1 selects a copy kernel
 * instead (up to 32 blocks per launch, the GPU accessing the pinned host memory
 * directly), faster per block but in competition with a concurrent decode step. */
int fs_pool_offload(fs_pool *pool, const int32_t *block_ids, const int32_t *host_slots,
                    int32_t n, void *stream);
int fs_pool_upload(fs_pool *pool, const int32_t *host_slots, const int32_t *block_ids,
                   int32_t n, void *stream);

/* ---- measurement and tuning helpers ---------------------------------------------- */

typedef enum fs_kernel_kind {
    FS_KERNEL_APPEND = 0,
    FS_KERNEL_ATTENTION = 1, /* partitioned attention with online softmax             */
    FS_KERNEL_COMBINE = 2,   /* merge of the partitions of one (job, head)            */
    FS_KERNEL_PREFILL = 3,           /* bulk KV write                                  */
    FS_KERNEL_PREFILL_ATTENTION = 4, /* prompt-phase attention                         */
    FS_KERNEL_PREFILL_PLAN = 5,      /* its work list                                  */
    FS_KERNEL_KINDS = 6
} fs_kernel_kind;

/* While enabled, every kernel launch carries a pair of HIP events on its stream that the
 * runtime stamps with the kernel's own start and end. */
int fs_profile_enable(fs_pool *pool, int32_t enable);
/* Waits for the recorded events; adds up milliseconds and launch counts per
 * fs_kernel_kind into total_ms[FS_KERNEL_KINDS], launches[FS_KERNEL_KINDS]
 * (host arrays), then forgets the records. */
int fs_profile_collect(fs_pool *pool, float *total_ms, int32_t *launches);

/* Named integer knobs for sweeps:
 *   "wgs_per_cu"       persistent attention workgroups per compute unit, 1..8; 0 = default:
 *                      for fs_decode_attention one per compute unit, of which a batch with
 *                      at least 8 steps of 64 tokens per wave uses 7 of every 8 (decided on
 *                      the device); for fs_decode_step 2 per compute unit;
 *   "max_workgroups"   cap on that grid, 0 = none;
 *   "swap_engine"      see fs_pool_offload;
 *   "append_in_attention"  fs_decode_step only.  0 (default): the attention kernel takes the
 *                      new tokens from k, v and leaves writing them into the pool to the launch
 *                      that follows it (extra workgroups of the combine pass); 1: it writes
 *                      them itself as it meets them.  Same pool bytes and same `out` either way;
 *   "merge_in_kernel"  0 (default): a (job, head) pair whose cache was split over several
 *                      waves is merged by a combine launch after the attention kernel;
 *                      1: by the attention kernel itself -- the last wave to finish its share
 *                      of such a pair merges it, no second launch.  Same arithmetic in the
 *                      same order, hence the same bits in `out`.
 * Readable also: "num_cus", "max_jobs_per_launch".  Unknown name or out-of-range value ->
 * FS_ERR_INVALID_ARG. */
int fs_pool_set_param(fs_pool *pool, const char *name, int32_t value);
int fs_pool_get_param(const fs_pool *pool, const char *name, int32_t *value);

/* Copies the attention kernel's last work plan to the host after waiting for
 * `stream`: step_base[num_jobs+1], the prefix sum over jobs of 64-token steps
 * (ceil(job_lens[j] / 64)) that the kernels split evenly over the waves.  Test
 * helper; num_jobs at most 1024 (the last launch slice of a larger batch). */
int fs_pool_last_plan(fs_pool *pool, int32_t num_jobs, int32_t *step_base, void *stream);

/* Plain streaming kernels of known size: a read of `bytes` from src and a copy of `bytes`
 * from src to dst, pointers the GPU can reach (device memory, or pinned host memory), 16-byte
 * aligned, bytes a multiple of 16, on `workgroups` workgroups of 256 threads.  They
 * give the practical HBM ceiling of the GPU at hand and the scale of the hardware
 * byte counters; the cache manager brings a batch's tables from pinned memory to the GPU
 * with the copy (fs_kvm_stage_batch).  sink: 16 writable device bytes. */
int fs_stream_read(const void *src, size_t bytes, void *sink, int32_t workgroups, void *stream);
int fs_stream_copy(void *dst, const void *src, size_t bytes, int32_t workgroups, void *stream);
/* fs_stream_read that waits for its kernel and reports the kernel's own duration in
 * microseconds in *kernel_us (host pointer), taken from events attached to the launch: the
 * span a profiler reports for the dispatch, and the way the duration of a profiled pool's
 * kernels is taken, so that the two compare like for like. */
int fs_stream_read_timed(const void *src, size_t bytes, void *sink, int32_t workgroups, void *stream,
                         float *kernel_us);

const char *fs_strerror(int status);
const char *fs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FASTSERVE_H */
