/*
 * CPU oracle for one decode iteration over per-job KV caches.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the GPU path and the
 * product never calls it; only the tests, the smoke check and the bench's
 * cpu_baseline leg may.
 *
 * What it computes (paper Section 2.2, "key-value cache" and Figure 3): in the
 * decoding phase each job contributes one new token; its key and value join
 * the job's cache, and the masked self-attention of that token uses the keys
 * and values of all tokens up to and including itself.  The paper names the
 * operator (Transformer masked self-attention) without printing a formula, so
 * this is the textbook scaled-dot-product definition, written out:
 *
 *     s_t        = scale * sum_d q[h][d] * K[t][h][d]          t = 0 .. L-1
 *     w_t        = exp(s_t - max_u s_u) / sum_u exp(s_u - max_u s_u)
 *     out[h][d]  = sum_t w_t * V[t][h][d]
 *
 * scale = 1/sqrt(D) unless the caller passes another value.  Block paging
 * (Section 2.2, block-grained allocation) is a storage matter and does not
 * exist here: a job's cache is one contiguous logical array K[t][h][d].
 *
 * All arithmetic is IEEE double; bf16, fp16 and fp32 inputs widen exactly.
 * (fp16 is the precision of the paper's own runs, Section 6.1.)
 * Single-threaded, no blocking, no reordering.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { FSO_BF16 = 0, FSO_F32 = 1, FSO_F64 = 2, FSO_F16 = 3 };

static size_t elem_size(int dtype)
{
    return (dtype == FSO_BF16 || dtype == FSO_F16) ? 2 : dtype == FSO_F32 ? 4 : 8;
}

/* exact widening of element i of a typed array */
static double load_elem(const void *base, int dtype, size_t i)
{
    if (dtype == FSO_BF16) {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    if (dtype == FSO_F16) {
        /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
        uint16_t h = ((const uint16_t *)base)[i];
        int e = (h >> 10) & 0x1f;
        double frac = (double)(h & 0x3ff) / 1024.0;
        double mag;
        if (e == 0)
            mag = ldexp(frac, -14);                 /* zero and subnormals */
        else if (e == 31)
            mag = (h & 0x3ff) ? NAN : INFINITY;
        else
            mag = ldexp(1.0 + frac, e - 15);
        return (h & 0x8000) ? -mag : mag;
    }
    if (dtype == FSO_F32)
        return (double)((const float *)base)[i];
    return ((const double *)base)[i];
}

/*
 * KV append of the decoding phase (Section 2.2): the new token's key and
 * value rows become row `len` of the job's logical cache (capacity > len).
 * A bit copy: no conversion.  k_new, v_new: [H][D].
 */
int fso_append(void *K, void *V, int dtype, long len, int H, int D,
               const void *k_new, const void *v_new)
{
    if (!K || !V || !k_new || !v_new || len < 0 || H <= 0 || D <= 0)
        return -1;
    size_t row = (size_t)H * (size_t)D * elem_size(dtype);
    memcpy((char *)K + (size_t)len * row, k_new, row);
    memcpy((char *)V + (size_t)len * row, v_new, row);
    return 0;
}

/*
 * Attention of one job's new token over its whole cache, heads [h0, h1).
 *   q: [H][D]   K, V: [L][H][D]   out: [H][D] doubles (rows h0..h1-1 written)
 *   weights: NULL or [H][L] doubles receiving w_t (rows h0..h1-1 written)
 *   scale <= 0 selects 1/sqrt(D).
 * L == 0 writes zeros (an empty cache attends to nothing).
 */
int fso_attention_job(const void *q, const void *K, const void *V, int dtype,
                      long L, int H, int D, double scale, int h0, int h1,
                      double *out, double *weights)
{
    if (!q || !out || L < 0 || H <= 0 || D <= 0 || h0 < 0 || h1 > H || h0 > h1)
        return -1;
    if (L > 0 && (!K || !V))
        return -1;
    if (scale <= 0.0)
        scale = 1.0 / sqrt((double)D);
    double *s = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    if (!s)
        return -2;
    for (int h = h0; h < h1; ++h) {
        double *o = out + (size_t)h * D;
        for (int d = 0; d < D; ++d)
            o[d] = 0.0;
        if (L == 0)
            continue;
        double smax = -INFINITY;
        for (long t = 0; t < L; ++t) {
            double dot = 0.0;
            for (int d = 0; d < D; ++d)
                dot += load_elem(q, dtype, (size_t)h * D + d) *
                       load_elem(K, dtype, ((size_t)t * H + h) * D + d);
            s[t] = scale * dot;
            if (s[t] > smax)
                smax = s[t];
        }
        double denom = 0.0;
        for (long t = 0; t < L; ++t) {
            s[t] = exp(s[t] - smax);
            denom += s[t];
        }
        for (long t = 0; t < L; ++t) {
            double w = s[t] / denom;
            if (weights)
                weights[(size_t)h * L + t] = w;
            for (int d = 0; d < D; ++d)
                o[d] += w * load_elem(V, dtype, ((size_t)t * H + h) * D + d);
        }
    }
    free(s);
    return 0;
}

/*
 * One whole decode step for a batch: append then attend, job by job.
 *   K[j], V[j]: logical caches with capacity >= lens_before[j] + 1 rows
 *   k_new, v_new, q: [J][H][D]     out: [J][H][D] doubles
 */
int fso_decode_step(void *const *K, void *const *V, const long *lens_before,
                    int J, int dtype, int H, int D, double scale,
                    const void *k_new, const void *v_new, const void *q,
                    double *out)
{
    size_t row = (size_t)H * (size_t)D;
    for (int j = 0; j < J; ++j) {
        const char *kn = (const char *)k_new + (size_t)j * row * elem_size(dtype);
        const char *vn = (const char *)v_new + (size_t)j * row * elem_size(dtype);
        const char *qj = (const char *)q + (size_t)j * row * elem_size(dtype);
        int rc = fso_append(K[j], V[j], dtype, lens_before[j], H, D, kn, vn);
        if (rc)
            return rc;
        rc = fso_attention_job(qj, K[j], V[j], dtype, lens_before[j] + 1, H, D,
                               scale, 0, H, out + (size_t)j * row, NULL);
        if (rc)
            return rc;
    }
    return 0;
}

/*
 * Initialization phase (paper Section 2.2, Figure 3, first iteration): all s
 * prompt tokens of a job are processed at once; token i's masked self-attention
 * sees the keys and values of tokens 0..i of the same prompt and nothing later.
 * Written out:
 *
 *     s_it       = scale * sum_d Q[i][h][d] * K[t][h][d]        0 <= t <= i
 *     w_it       = exp(s_it - max_{u<=i} s_iu) / sum_{u<=i} exp(s_iu - max ...)
 *     out[i][h]  = sum_{t<=i} w_it * V[t][h][:]
 *
 *   Q, K, V: [s][H][D]   out: [s][H][D] doubles, heads [h0, h1) written.
 */
int fso_prefill_attention_job(const void *Q, const void *K, const void *V, int dtype,
                              long s, int H, int D, double scale, int h0, int h1,
                              double *out)
{
    if (s < 0 || H <= 0 || D <= 0 || h0 < 0 || h1 > H || h0 > h1)
        return -1;
    if (s == 0)
        return 0;
    if (!Q || !K || !V || !out)
        return -1;
    if (scale <= 0.0)
        scale = 1.0 / sqrt((double)D);
    double *sc = (double *)malloc(sizeof(double) * (size_t)s);
    if (!sc)
        return -2;
    for (long i = 0; i < s; ++i) {
        for (int h = h0; h < h1; ++h) {
            double *o = out + ((size_t)i * H + h) * D;
            double smax = -INFINITY;
            for (long t = 0; t <= i; ++t) {
                double dot = 0.0;
                for (int d = 0; d < D; ++d)
                    dot += load_elem(Q, dtype, ((size_t)i * H + h) * D + d) *
                           load_elem(K, dtype, ((size_t)t * H + h) * D + d);
                sc[t] = scale * dot;
                if (sc[t] > smax)
                    smax = sc[t];
            }
            double denom = 0.0;
            for (long t = 0; t <= i; ++t) {
                sc[t] = exp(sc[t] - smax);
                denom += sc[t];
            }
            for (int d = 0; d < D; ++d)
                o[d] = 0.0;
            for (long t = 0; t <= i; ++t) {
                double w = sc[t] / denom;
                for (int d = 0; d < D; ++d)
                    o[d] += w * load_elem(V, dtype, ((size_t)t * H + h) * D + d);
            }
        }
    }
    free(sc);
    return 0;
}
