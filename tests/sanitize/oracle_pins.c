/*
 * Runs the C oracle (oracle/fs_oracle.c, compiled with -fsanitize=address,undefined) through its
 * pins on small seeded inputs: a one-token cache returns its value row, identical keys give the
 * mean of the values, the weights sum to one, the whole step equals append + attention, and row i
 * of the prompt-phase function equals the decode function on the prompt cut after token i.  Every
 * buffer is sized exactly, so that any access past an end is reported.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int fso_append(void *K, void *V, int dtype, long len, int H, int D, const void *k_new, const void *v_new);
int fso_attention_job(const void *q, const void *K, const void *V, int dtype, long L, int H, int D, double scale,
                      int h0, int h1, double *out, double *weights);
int fso_decode_step(void *const *K, void *const *V, const long *lens_before, int J, int dtype, int H, int D,
                    double scale, const void *k_new, const void *v_new, const void *q, double *out);
int fso_prefill_attention_job(const void *Q, const void *K, const void *V, int dtype, long s, int H, int D,
                              double scale, int h0, int h1, double *out);

#define CHECK(cond)                                                                   \
    do {                                                                              \
        if (!(cond)) {                                                                \
            fprintf(stderr, "oracle_pins.c:%d: check failed: %s\n", __LINE__, #cond); \
            return 1;                                                                 \
        }                                                                             \
    } while (0)

static uint64_t rng_state = 0x2305059200000001ull;
static double uniform(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}
static uint16_t bf16_of(double x) /* truncation is enough: the pins hold for any stored value */
{
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}
static double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}
static uint16_t *random_rows(long n, int H, int D)
{
    uint16_t *a = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)(n > 0 ? n : 1) * H * D);
    for (long i = 0; a && i < n * H * D; ++i) a[i] = bf16_of(2.0 * uniform() - 1.0);
    return a;
}

int main(void)
{
    enum { H = 3, D = 8, BF16 = 0 };
    for (int dtype_case = 0; dtype_case < 2; ++dtype_case) {
        const int dtype = dtype_case == 0 ? BF16 : 3; /* bf16 and f16 storage share the 2-byte buffers */
        for (long L = 1; L <= 33; L += 8) {
            uint16_t *q = random_rows(1, H, D), *Kc = random_rows(L, H, D), *Vc = random_rows(L, H, D);
            double *out = (double *)malloc(sizeof(double) * H * D), *w = (double *)malloc(sizeof(double) * H * L);
            CHECK(q && Kc && Vc && out && w);
            CHECK(fso_attention_job(q, Kc, Vc, dtype, L, H, D, 0.0, 0, H, out, w) == 0);
            for (int h = 0; h < H; ++h) { /* the weights of a head sum to one */
                double sum = 0;
                for (long t = 0; t < L; ++t) sum += w[(size_t)h * L + t];
                CHECK(fabs(sum - 1.0) < 1e-12);
            }
            if (L == 1 && dtype == BF16) /* a one-token cache returns its value row */
                for (int i = 0; i < H * D; ++i) CHECK(out[i] == bf16_to_double(Vc[i]));
            /* identical keys: every weight 1/L, the output the mean of the values */
            for (long t = 1; t < L; ++t) memcpy(Kc + (size_t)t * H * D, Kc, sizeof(uint16_t) * H * D);
            CHECK(fso_attention_job(q, Kc, Vc, BF16, L, H, D, 0.0, 0, H, out, NULL) == 0);
            for (int i = 0; i < H * D; ++i) {
                double mean = 0;
                for (long t = 0; t < L; ++t) mean += bf16_to_double(Vc[(size_t)t * H * D + i]);
                CHECK(fabs(out[i] - mean / L) < 1e-12);
            }
            /* heads outside [h0, h1) are left alone; an empty cache gives zeros */
            for (int i = 0; i < H * D; ++i) out[i] = 7.0;
            CHECK(fso_attention_job(q, Kc, Vc, BF16, L, H, D, 0.0, 1, 2, out, NULL) == 0);
            CHECK(out[0] == 7.0 && out[2 * D] == 7.0);
            CHECK(fso_attention_job(q, NULL, NULL, BF16, 0, H, D, 0.0, 0, H, out, NULL) == 0 && out[0] == 0.0);
            free(q), free(Kc), free(Vc), free(out), free(w);
        }
    }
    { /* whole step = append + attention; prompt row i = decode over the prompt cut after token i */
        enum { J = 3 };
        const long lens[J] = {0, 5, 16};
        void *Kp[J], *Vp[J];
        for (int j = 0; j < J; ++j) {
            uint16_t *k = random_rows(lens[j] + 1, H, D), *v = random_rows(lens[j] + 1, H, D); /* capacity exactly len + 1 */
            CHECK(k && v);
            Kp[j] = k, Vp[j] = v;
        }
        uint16_t *kn = random_rows(J, H, D), *vn = random_rows(J, H, D), *q = random_rows(J, H, D);
        double *out = (double *)malloc(sizeof(double) * J * H * D), *one = (double *)malloc(sizeof(double) * H * D);
        CHECK(kn && vn && q && out && one);
        CHECK(fso_decode_step(Kp, Vp, lens, J, BF16, H, D, 0.0, kn, vn, q, out) == 0);
        for (int j = 0; j < J; ++j) {
            CHECK(memcmp((uint16_t *)Kp[j] + (size_t)lens[j] * H * D, kn + (size_t)j * H * D, sizeof(uint16_t) * H * D) == 0);
            CHECK(fso_attention_job(q + (size_t)j * H * D, Kp[j], Vp[j], BF16, lens[j] + 1, H, D, 0.0, 0, H, one, NULL) == 0);
            CHECK(memcmp(one, out + (size_t)j * H * D, sizeof(double) * H * D) == 0);
        }
        const long s = 17;
        uint16_t *Q = random_rows(s, H, D);
        double *po = (double *)malloc(sizeof(double) * s * H * D);
        CHECK(Q && po);
        CHECK(fso_prefill_attention_job(Q, Kp[2], Vp[2], BF16, s, H, D, 0.0, 0, H, po) == 0);
        for (long i = 0; i < s; ++i) {
            CHECK(fso_attention_job(Q + (size_t)i * H * D, Kp[2], Vp[2], BF16, i + 1, H, D, 0.0, 0, H, one, NULL) == 0);
            for (int x = 0; x < H * D; ++x) CHECK(fabs(one[x] - po[(size_t)i * H * D + x]) < 1e-12);
        }
        for (int j = 0; j < J; ++j) free(Kp[j]), free(Vp[j]);
        free(kn), free(vn), free(q), free(out), free(one), free(Q), free(po);
    }
    printf("oracle pins ok\n");
    return 0;
}
