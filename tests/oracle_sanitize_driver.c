/*
 * Drives every entry point of oracle/detonation_oracle.c over odd shapes so that a build with
 * -fsanitize=address,undefined (no OpenMP) shows any out-of-bounds access, misaligned access,
 * signed overflow or leak in the checker itself.  Every buffer is allocated at exactly the
 * size the entry point documents, so an access one element past it is reported.
 * Test infrastructure: compiled and run only by tests/test_oracle_pins.py.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t chunk, topk, scheme;
    uint32_t flags;
    float decay, lr, weight_decay;
    uint64_t seed, step;
} orc_config;

typedef struct {
    float beta1, beta2, eps;
    int32_t amsgrad;
    uint64_t step;
} orc_adamw;

int orc_dct_matrix(int32_t s, double *D);
int orc_fold(const orc_config *, int64_t, const void *, int, const float *, float *);
int orc_transform(const orc_config *, int64_t, const float *, float *);
int orc_select(const orc_config *, int64_t, int64_t, const float *, int32_t *);
int orc_extract(const orc_config *, int64_t, const float *, const float *, const int32_t *,
                float *, float *);
int orc_extract_q(const orc_config *, int64_t, const float *, const float *, const int32_t *, int,
                  uint16_t *, float *);
int orc_presign(const orc_config *, int64_t, int32_t, const int32_t *, int64_t, const float *,
                int64_t, float *);
int orc_presign_q(const orc_config *, int64_t, int32_t, const int32_t *, int64_t,
                  const uint16_t *, int, int64_t, float *);
int64_t orc_ternary_words(const orc_config *, int64_t);
int orc_encode_ternary(const orc_config *, int64_t, const float *, uint32_t *);
int orc_decode_ternary(const orc_config *, int64_t, const uint32_t *, float *);
int orc_presign_t(const orc_config *, int64_t, int32_t, const int32_t *, int64_t,
                  const uint32_t *, int64_t, float *);
int orc_compress(const orc_config *, int64_t, const void *, int, float *, int32_t *, float *,
                 float *);
int orc_update(const orc_config *, int64_t, const float *, void *, int);
int orc_adamw_update(const orc_config *, const orc_adamw *, int64_t, const float *, void *, int,
                     float *, float *, float *);
int orc_decompress_step(const orc_config *, int64_t, int32_t, const int32_t *, int64_t,
                        const float *, int64_t, void *, int, float *);
uint16_t orc_double_to_bf16(double);
uint16_t orc_float_to_f16(float);
float orc_f16_to_float(uint16_t);

static uint32_t lcg_state = 12345u;
static float rnd(void)
{
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return ((float)(lcg_state >> 8) / 8388608.0f - 1.0f) * 1e-3f;
}

#define NEED(call)                                                                  \
    do {                                                                            \
        int rc_ = (call);                                                           \
        if (rc_ != 0) {                                                             \
            fprintf(stderr, "%s -> %d (s=%d k=%d scheme=%d)\n", #call, rc_, s, k, scheme); \
            return 1;                                                               \
        }                                                                           \
    } while (0)

static int one_case(int s, int k, int scheme, int dct, int64_t n, int R, int bf16)
{
    orc_config cfg = {s, k, scheme, 1u | (dct ? 2u : 0u), 0.9f, 1e-3f, 0.01f, 77u,
                      (uint64_t)(s + k)};
    const int64_t C = (n + s - 1) / s, E = C * k;
    float *m = malloc(sizeof(float) * (size_t)(n ? n : 1));
    float *m1 = malloc(sizeof(float) * (size_t)(n ? n : 1));
    float *mn = malloc(sizeof(float) * (size_t)(n ? n : 1));
    void *g = malloc((bf16 ? 2 : 4) * (size_t)(n ? n : 1));
    void *th = malloc((bf16 ? 2 : 4) * (size_t)(n ? n : 1));
    float *coeff = malloc(sizeof(float) * (size_t)(C * s + 1));
    int32_t *idx = malloc(sizeof(int32_t) * (size_t)(R * E + 1));
    float *val = malloc(sizeof(float) * (size_t)(R * E + 1));
    uint16_t *vq = malloc(sizeof(uint16_t) * (size_t)(R * E + 1));
    float *y = malloc(sizeof(float) * (size_t)(n ? n : 1));
    float *ea = calloc((size_t)(n ? n : 1), sizeof(float));
    float *es = calloc((size_t)(n ? n : 1), sizeof(float));
    float *em = calloc((size_t)(n ? n : 1), sizeof(float));
    for (int64_t i = 0; i < n; ++i) {
        m[i] = rnd();
        if (bf16) {
            ((uint16_t *)g)[i] = orc_double_to_bf16((double)rnd());
            ((uint16_t *)th)[i] = orc_double_to_bf16((double)rnd() * 20.0);
        } else {
            ((float *)g)[i] = rnd();
            ((float *)th)[i] = rnd() * 20.0f;
        }
    }
    /* the steps one by one */
    NEED(orc_fold(&cfg, n, g, bf16, m, m1));
    NEED(orc_transform(&cfg, n, m1, coeff));
    NEED(orc_select(&cfg, C, 1000003, coeff, idx));
    NEED(orc_extract(&cfg, n, m1, coeff, idx, val, mn));
    NEED(orc_extract_q(&cfg, n, m1, coeff, idx, 1, vq, mn));
    NEED(orc_extract_q(&cfg, n, m1, coeff, idx, 2, vq, mn));
    /* R replicas of the same payload, side by side */
    for (int r = 1; r < R; ++r) {
        memcpy(idx + r * E, idx, sizeof(int32_t) * (size_t)E);
        memcpy(val + r * E, val, sizeof(float) * (size_t)E);
        memcpy(vq + r * E, vq, sizeof(uint16_t) * (size_t)E);
    }
    NEED(orc_presign(&cfg, n, R, idx, E, val, E, y));
    NEED(orc_presign_q(&cfg, n, R, idx, E, vq, 2, E, y));
    if (scheme != 0) NEED(orc_presign(&cfg, n, R, NULL, 0, val, E, y));
    /* ternary words */
    const int64_t W = orc_ternary_words(&cfg, n);
    uint32_t *words = malloc(sizeof(uint32_t) * (size_t)(R * W + 1));
    NEED(orc_encode_ternary(&cfg, n, val, words));
    for (int r = 1; r < R; ++r) memcpy(words + r * W, words, sizeof(uint32_t) * (size_t)W);
    NEED(orc_decode_ternary(&cfg, n, words, val));
    NEED(orc_presign_t(&cfg, n, R, idx, E, words, W, y));
    /* updates */
    orc_adamw opt = {0.9f, 0.95f, 1e-8f, 1, 3u};
    NEED(orc_update(&cfg, n, y, th, bf16));
    NEED(orc_adamw_update(&cfg, &opt, n, y, th, bf16, ea, es, em));
    /* the two composites */
    NEED(orc_compress(&cfg, n, g, bf16, m, idx, val, coeff));
    NEED(orc_compress(&cfg, n, g, bf16, m, NULL, val, NULL));
    for (int r = 1; r < R; ++r) memcpy(val + r * E, val, sizeof(float) * (size_t)E);
    NEED(orc_decompress_step(&cfg, n, R, idx, E, val, E, th, bf16, y));
    NEED(orc_decompress_step(&cfg, n, R, idx, E, val, E, th, bf16, NULL));
    free(words); free(em); free(es); free(ea); free(y); free(vq); free(val); free(idx);
    free(coeff); free(th); free(g); free(mn); free(m1); free(m);
    return 0;
}

int main(void)
{
    static const int shapes[][2] = {{1, 1}, {2, 1}, {3, 2}, {7, 7}, {16, 2}, {32, 1}, {32, 16},
                                    {64, 8}, {64, 32}, {65, 7}, {96, 12}, {128, 64}, {192, 24},
                                    {200, 100}, {255, 254}, {256, 1}, {256, 256}};
    int cases = 0;
    for (size_t i = 0; i < sizeof(shapes) / sizeof(shapes[0]); ++i) {
        const int s = shapes[i][0], k = shapes[i][1];
        for (int scheme = 0; scheme < 3; ++scheme) {
            for (int dct = 0; dct < 2; ++dct) {
                if (scheme == 0 && dct) continue;
                /* whole chunks, a ragged tail, a shard shorter than one chunk */
                const int64_t lens[3] = {(int64_t)s * 5, (int64_t)s * 3 + (s + 1) / 2, (s + 2) / 3};
                for (int l = 0; l < 3; ++l) {
                    if (one_case(s, k, scheme, dct, lens[l], 1 + (int)(i % 3), (int)((i + l) % 2)))
                        return 1;
                    ++cases;
                }
            }
        }
    }
    /* n = 0 is a no-op everywhere */
    if (one_case(64, 8, 0, 0, 0, 2, 0)) return 1;
    /* conversions over every 16-bit pattern */
    double acc = 0.0;
    for (uint32_t b = 0; b < 65536u; ++b) {
        const float f = orc_f16_to_float((uint16_t)b);
        if (f == f) acc += (double)orc_float_to_f16(f) + (double)orc_double_to_bf16((double)f);
    }
    double *D = malloc(sizeof(double) * 256 * 256);
    if (orc_dct_matrix(256, D)) return 1;
    free(D);
    printf("sanitize driver: %d cases clean (%.0f)\n", cases + 1, acc);
    return 0;
}
