/*
 * A plain C caller of the library: no Python, no tensor library, only the two public headers
 * and the HIP runtime for device memory.  `client host` exercises what needs no GPU (version,
 * error strings, argument checks, the scheduler); `client gpu` runs a tiny decode step and
 * checks it against closed forms: a one-token cache returns its value row, identical keys
 * give the mean of the values (bf16 inputs chosen so that both are exact in fp32).
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "fastserve.h"
#include "fastserve_sched.h"

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            return 1;                                                      \
        }                                                                  \
    } while (0)

static uint16_t bf16_of(float f) /* exact for the small integers and halves used here */
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}

static int host_checks(void)
{
    CHECK(fs_version() != NULL && strlen(fs_version()) > 0);
    CHECK(strcmp(fs_strerror(FS_OK), fs_strerror(FS_ERR_INVALID_ARG)) != 0);
    fs_pool *pool = NULL;
    CHECK(fs_pool_create(NULL, &pool) == FS_ERR_INVALID_ARG);
    fs_pool_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.dtype = FS_BF16; cfg.num_heads = 2; cfg.head_dim = 96; cfg.block_size = 16; cfg.num_blocks = 4;
    CHECK(fs_pool_create(&cfg, &pool) == FS_ERR_UNSUPPORTED);      /* head_dim 96 is not built */
    cfg.head_dim = 128; cfg.num_blocks = 0;
    CHECK(fs_pool_create(&cfg, &pool) == FS_ERR_INVALID_ARG);
    CHECK(fs_kv_append(NULL, NULL, 0, NULL, 1, NULL, NULL, NULL) == FS_ERR_INVALID_ARG);

    fs_sched *s = NULL;
    CHECK(fs_sched_create(4, 1.0, 1, 100.0, 2, &s) == FS_OK && s != NULL);
    int32_t queue = 0;
    CHECK(fs_sched_add_job(s, 7, 0.5, 1.0, &queue) == FS_OK && queue == 1);   /* fits the first quantum */
    CHECK(fs_sched_add_job(s, 8, 3.0, 1.0, &queue) == FS_OK && queue == 3);   /* skip-joins: 1, 2, 4 >= 3 */
    CHECK(fs_sched_add_job(s, 7, 1.0, 1.0, &queue) != FS_OK);                 /* duplicate id */
    int64_t batch[2];
    int32_t n = 0;
    CHECK(fs_sched_schedule(s, batch, 2, &n) == FS_OK && n == 2 && batch[0] == 7 && batch[1] == 8);
    int64_t done[1] = {7};
    CHECK(fs_sched_complete_iteration(s, batch, 2, 3.0, done, 1) == FS_OK);
    CHECK(fs_sched_num_jobs(s) == 1);
    CHECK(fs_sched_destroy(s) == FS_OK);
    printf("host checks ok (%s)\n", fs_version());
    return 0;
}

static int gpu_checks(void)
{
    enum { H = 2, D = 128, B = 16, NB = 4, J = 2 };
    fs_pool_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.dtype = FS_BF16; cfg.num_heads = H; cfg.head_dim = D; cfg.block_size = B; cfg.num_blocks = NB;
    fs_pool *pool = NULL;
    CHECK(fs_pool_create(&cfg, &pool) == FS_OK);
    CHECK(fs_pool_block_bytes(pool) == (size_t)2 * H * B * D * 2);

    /* job 0: empty cache, one new token -> out = its value row.
       job 1: three cached tokens with identical keys plus a new token with the same key ->
       out = mean of the four value rows (values are small integers: exact). */
    static uint16_t k_new[J][H][D], v_new[J][H][D], q[J][H][D];
    static uint16_t kc[3][H][D], vc[3][H][D];
    for (int h = 0; h < H; ++h)
        for (int d = 0; d < D; ++d) {
            const float key = (float)((d % 5) - 2) * 0.5f;
            k_new[0][h][d] = bf16_of((float)(d % 3)); v_new[0][h][d] = bf16_of((float)(h * 7 + d % 11) - 4.0f);
            q[0][h][d] = bf16_of(1.0f); q[1][h][d] = bf16_of((float)(d % 2));
            k_new[1][h][d] = bf16_of(key); v_new[1][h][d] = bf16_of(8.0f);
            for (int t = 0; t < 3; ++t) { kc[t][h][d] = bf16_of(key); vc[t][h][d] = bf16_of((float)(4 * t + (d % 2) * 4)); }
        }
    int32_t table[J][2] = {{2, -1}, {3, -1}}, lens_before[J] = {0, 3}, lens_after[J] = {1, 4};

    void *d_k, *d_v, *d_q, *d_kc, *d_vc, *d_table, *d_lb, *d_la, *d_offs, *d_starts;
    float *d_out;
    CHECK(hipMalloc(&d_k, sizeof k_new) == hipSuccess && hipMalloc(&d_v, sizeof v_new) == hipSuccess);
    CHECK(hipMalloc(&d_q, sizeof q) == hipSuccess && hipMalloc(&d_kc, sizeof kc) == hipSuccess);
    CHECK(hipMalloc(&d_vc, sizeof vc) == hipSuccess && hipMalloc(&d_table, sizeof table) == hipSuccess);
    CHECK(hipMalloc(&d_lb, sizeof lens_before) == hipSuccess && hipMalloc(&d_la, sizeof lens_after) == hipSuccess);
    CHECK(hipMalloc(&d_offs, 2 * sizeof(int32_t)) == hipSuccess && hipMalloc(&d_starts, sizeof(int32_t)) == hipSuccess);
    CHECK(hipMalloc((void **)&d_out, sizeof(float) * J * H * D) == hipSuccess);
    CHECK(hipMemcpy(d_k, k_new, sizeof k_new, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_v, v_new, sizeof v_new, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_q, q, sizeof q, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_kc, kc, sizeof kc, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_vc, vc, sizeof vc, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_table, table, sizeof table, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_lb, lens_before, sizeof lens_before, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_la, lens_after, sizeof lens_after, hipMemcpyHostToDevice) == hipSuccess);
    int32_t offs[2] = {0, 3}, starts[1] = {0};
    CHECK(hipMemcpy(d_offs, offs, sizeof offs, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_starts, starts, sizeof starts, hipMemcpyHostToDevice) == hipSuccess);

    /* job 1's three cached tokens through the bulk write (its table row only) */
    CHECK(fs_kv_prefill(pool, (const int32_t *)d_table + 2, 2, d_starts, d_offs, 1, 3, d_kc, d_vc, NULL) == FS_OK);
    CHECK(fs_kv_append(pool, d_table, 2, d_lb, J, d_k, d_v, NULL) == FS_OK);
    CHECK(fs_decode_attention(d_q, pool, d_table, 2, d_la, J, 0, d_out, NULL) == FS_OK);
    CHECK(fs_pool_check(pool, NULL) == FS_OK);
    static float out[J][H][D];
    CHECK(hipMemcpy(out, d_out, sizeof out, hipMemcpyDeviceToHost) == hipSuccess);
    for (int h = 0; h < H; ++h)
        for (int d = 0; d < D; ++d) {
            const float want0 = (float)(h * 7 + d % 11) - 4.0f;
            const float want1 = (0.0f + 4.0f + 8.0f + 3.0f * (float)((d % 2) * 4) + 8.0f) / 4.0f;
            CHECK(out[0][h][d] == want0);
            CHECK(fabsf(out[1][h][d] - want1) <= 1e-6f);
        }
    /* the same step through the fused entry point on fresh blocks */
    int32_t table2[J][2] = {{0, -1}, {1, -1}};
    CHECK(hipMemcpy(d_table, table2, sizeof table2, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(fs_kv_prefill(pool, (const int32_t *)d_table + 2, 2, d_starts, d_offs, 1, 3, d_kc, d_vc, NULL) == FS_OK);
    CHECK(fs_decode_step(pool, d_table, 2, d_lb, J, d_k, d_v, d_q, 0, d_out, NULL) == FS_OK);
    CHECK(fs_pool_check(pool, NULL) == FS_OK);
    static float out2[J][H][D];
    CHECK(hipMemcpy(out2, d_out, sizeof out2, hipMemcpyDeviceToHost) == hipSuccess);
    CHECK(memcmp(out2[0], out[0], sizeof out[0]) == 0);
    for (int h = 0; h < H; ++h)
        for (int d = 0; d < D; ++d) CHECK(fabsf(out2[1][h][d] - out[1][h][d]) <= 1e-6f);
    /* a table entry outside the pool raises the flag instead of a fault */
    int32_t bad[J][2] = {{99, -1}, {1, -1}};
    CHECK(hipMemcpy(d_table, bad, sizeof bad, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(fs_decode_attention(d_q, pool, d_table, 2, d_la, J, 0, d_out, NULL) == FS_OK);
    CHECK(fs_pool_check(pool, NULL) == FS_ERR_BAD_TABLE);
    CHECK(fs_pool_destroy(pool) == FS_OK);
    printf("gpu checks ok\n");
    return 0;
}

int main(int argc, char **argv)
{
    if (argc == 2 && strcmp(argv[1], "host") == 0) return host_checks();
    if (argc == 2 && strcmp(argv[1], "gpu") == 0) return host_checks() || gpu_checks();
    fprintf(stderr, "usage: client host|gpu\n");
    return 2;
}
