/*
 * CPU oracle for the FlexDeMo / DeMo-SGD optimizer step (arXiv 2502.06728).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously
 * correct statement of what one optimizer step computes on one flat shard, used
 * only to check the GPU library and as a timed CPU baseline.  It shares no code
 * with the HIP path and must never be called from it.
 *
 * What it follows
 *   Algorithm 1 of the paper, one shard, one rank:
 *     m  <- beta*m + Delta                      (momentum accumulate)
 *     q  <- ExtractFastComponents(m, s, k)      (chunked DCT-II, keep k per chunk)
 *     m  <- m - q                               (remove q from m)
 *     Q  <- Synchronize(q, R)                   (here: R payloads handed in, averaged)
 *     th <- th - eta*Q                          (parameter update)
 *   Section "Methods": the fast components are computed with the DCT-II.
 *   Section "Replication Schemes": Striding keeps every n-th index, Random keeps
 *   randomly chosen indices reproducible from a shared seed, neither transmits
 *   indices and neither works on DCT chunks unless asked to.
 *   Section "Overall Setup" and Appendix B: the sign function (torch.sign, so
 *   sign(0)=0) is optional; compression rate is k/s.
 *
 * Conventions
 *   State is kept at storage precision (momentum fp32, payload values fp32,
 *   indices int32, parameters fp32 or bf16).  All arithmetic between two stored
 *   quantities is done in double and rounded once when stored.
 *   D is the orthonormal DCT-II matrix  D[j][n] = a_j cos(pi (2n+1) j / (2s)),
 *   a_0 = sqrt(1/s), a_j = sqrt(2/s); its inverse is its transpose.
 *   The shard is cut into C = ceil(n/s) chunks of s consecutive elements; the last
 *   chunk is zero-extended and its pad positions are never written back.
 *
 * Parity pins (tests/, -m "not gpu"): D*D^T = I, agreement with scipy's
 * orthonormal DCT-II, Parseval, k = s lossless, energy bookkeeping of the residual,
 * brute-force best-k-subset on tiny chunks, hand-built ties, reduction to textbook
 * SGD with momentum, exhaustive bf16 rounding, closed-form Striding sets, Random
 * index statistics.  The paper prints no worked numeric example, so end-to-end
 * values are "parity unpinned" by the paper itself; the pins above are what there is.
 *
 * OpenMP is used only to run independent chunks side by side (for the timed
 * baseline); it changes no arithmetic and no order inside a chunk.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static const double ORC_PI = 3.14159265358979323846264338327950288;

enum { ORC_OK = 0, ORC_ERR_NULL = 1, ORC_ERR_BAD_CONFIG = 2 };
enum { ORC_SCHEME_TOPK = 0, ORC_SCHEME_STRIDE = 1, ORC_SCHEME_RANDOM = 2 };
enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F16 = 2 };
#define ORC_FLAG_SIGN 1u
#define ORC_FLAG_DCT 2u

typedef struct {
    int32_t chunk;        /* s */
    int32_t topk;         /* k */
    int32_t scheme;       /* ORC_SCHEME_* */
    uint32_t flags;       /* ORC_FLAG_* */
    float decay;          /* beta */
    float lr;             /* eta */
    float weight_decay;   /* lambda (decoupled) */
    uint64_t seed;        /* Random scheme: shared by all replicas */
    uint64_t step;        /* Striding offset / Random stream */
} orc_config;

/* ------------------------------------------------------------------ helpers */

static int orc_check(const orc_config *cfg)
{
    if (!cfg) return ORC_ERR_NULL;
    if (cfg->chunk < 1 || cfg->chunk > 256) return ORC_ERR_BAD_CONFIG;
    if (cfg->topk < 1 || cfg->topk > cfg->chunk) return ORC_ERR_BAD_CONFIG;
    if (cfg->scheme < 0 || cfg->scheme > 2) return ORC_ERR_BAD_CONFIG;
    return ORC_OK;
}

/* Top-k always works on DCT coefficients; Striding and Random work on the raw
 * momentum unless the DCT flag asks for the coefficient-domain variant. */
static int orc_uses_dct(const orc_config *cfg)
{
    return cfg->scheme == ORC_SCHEME_TOPK || (cfg->flags & ORC_FLAG_DCT) != 0;
}

int orc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

static float bf16_bits_to_float(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* Round a double to the nearest bf16 (8-bit significand), ties to even, in one
 * rounding.  Valid for finite values whose result is a normal bf16 or zero, which
 * is all the parameter update produces. */
uint16_t orc_double_to_bf16(double v)
{
    if (v == 0.0) return signbit(v) ? 0x8000u : 0u;
    uint64_t u;
    memcpy(&u, &v, 8);
    /* a double has 52 fraction bits, bf16 keeps 7: drop the low 45 */
    uint64_t lsb = (u >> 45) & 1u;
    u += ((1ull << 44) - 1ull) + lsb;
    u &= ~((1ull << 45) - 1ull);
    double r;
    memcpy(&r, &u, 8);
    float f = (float)r; /* exact: r has 8 significant bits */
    uint32_t w;
    memcpy(&w, &f, 4);
    return (uint16_t)(w >> 16);
}

static double load_elem(const void *p, int dtype, int64_t i)
{
    if (dtype == ORC_BF16) return (double)bf16_bits_to_float(((const uint16_t *)p)[i]);
    return (double)((const float *)p)[i];
}

/* ---------------------------------------------- 16-bit transfer formats */

/* fp32 -> IEEE half, round to nearest even, subnormals kept, overflow to infinity. */
uint16_t orc_float_to_f16(float f)
{
    uint32_t x;
    memcpy(&x, &f, 4);
    const uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    const uint32_t ax = x & 0x7FFFFFFFu;
    if (ax >= 0x7F800000u) return (uint16_t)(sign | 0x7C00u | ((ax > 0x7F800000u) ? 0x200u : 0u));
    if (ax >= 0x477FF000u) return (uint16_t)(sign | 0x7C00u);   /* >= 65520 rounds to infinity */
    if (ax < 0x38800000u) {
        /* below 2^-14: the result is a multiple of 2^-24; rint() rounds to nearest even */
        const double units = rint((double)fabsf(f) * 16777216.0);
        return (uint16_t)(sign | (uint16_t)units);               /* 1024 is the smallest normal */
    }
    const uint32_t mant = ax & 0x7FFFFFu;
    uint32_t half = (((ax >> 23) - 127u + 15u) << 10) | (mant >> 13);
    const uint32_t rem = mant & 0x1FFFu;
    if (rem > 0x1000u || (rem == 0x1000u && (half & 1u))) ++half;  /* a carry moves the exponent */
    return (uint16_t)(sign | half);
}

float orc_f16_to_float(uint16_t h)
{
    const int e = (h >> 10) & 0x1F, m = h & 0x3FF;
    double v;
    if (e == 0) v = ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    return (float)((h & 0x8000u) ? -v : v);
}

/* Transfer-dtype round trip of one payload value: what the receiver decodes.
 * (Appendix B, "Communication Floating Point Data Type": fp32 or a 16-bit format.) */
static float transfer_decode(int val_dtype, uint16_t bits)
{
    return val_dtype == ORC_F16 ? orc_f16_to_float(bits) : bf16_bits_to_float(bits);
}

static uint16_t transfer_encode(int val_dtype, float v)
{
    return val_dtype == ORC_F16 ? orc_float_to_f16(v) : orc_double_to_bf16((double)v);
}

/* defined further down; used by the quantised-payload variants above it */
int orc_presign(const orc_config *cfg, int64_t n, int32_t R, const int32_t *idx,
                int64_t idx_replica_stride, const float *val, int64_t val_replica_stride,
                float *y);

/* ------------------------------------------------------- DCT-II matrix (S1) */

/* D[j*s + n], orthonormal DCT-II of length s. */
int orc_dct_matrix(int32_t s, double *D)
{
    if (!D) return ORC_ERR_NULL;
    if (s < 1) return ORC_ERR_BAD_CONFIG;
    for (int j = 0; j < s; ++j) {
        double a = (j == 0) ? sqrt(1.0 / s) : sqrt(2.0 / s);
        for (int n = 0; n < s; ++n)
            D[(size_t)j * s + n] = a * cos(ORC_PI * (double)((2 * n + 1) * j) / (2.0 * s));
    }
    return ORC_OK;
}

/* --------------------------------------- Algorithm 1, momentum accumulate */

/* m1[i] = fl32(beta*m[i] + g[i]) */
int orc_fold(const orc_config *cfg, int64_t n, const void *grad, int grad_dtype,
             const float *m, float *m1)
{
    int rc = orc_check(cfg);
    if (rc) return rc;
    if (n > 0 && (!grad || !m || !m1)) return ORC_ERR_NULL;
    const double beta = (double)cfg->decay;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        m1[i] = (float)(beta * (double)m[i] + load_elem(grad, grad_dtype, i));
    return ORC_OK;
}

/* ------------------------------- ExtractFastComponents: chunked transform */

/* coeff[c*s + j] = fl32( sum_n D[j][n] * x[c*s + n] ), x read as 0 beyond n.
 * In the identity domain (no DCT) coeff is x itself, zero-extended. */
int orc_transform(const orc_config *cfg, int64_t n, const float *x, float *coeff)
{
    int rc = orc_check(cfg);
    if (rc) return rc;
    if (n > 0 && (!x || !coeff)) return ORC_ERR_NULL;
    const int s = cfg->chunk;
    const int64_t C = (n + s - 1) / s;
    if (!orc_uses_dct(cfg)) {
        for (int64_t i = 0; i < C * s; ++i) coeff[i] = (i < n) ? x[i] : 0.0f;
        return ORC_OK;
    }
    double *D = (double *)malloc(sizeof(double) * s * s);
    orc_dct_matrix(s, D);
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < C; ++c) {
        for (int j = 0; j < s; ++j) {
            double acc = 0.0;
            for (int t = 0; t < s; ++t) {
                int64_t i = c * s + t;
                double xv = (i < n) ? (double)x[i] : 0.0;
                acc += D[(size_t)j * s + t] * xv;
            }
            coeff[c * s + j] = (float)acc;
        }
    }
    free(D);
    return ORC_OK;
}

/* ------------------------------------------------ counter-based generator */

/* The Random scheme needs the same indices on every replica from a shared seed.
 * Specification (implemented independently by the GPU library):
 *   mix64 is the 64-bit finaliser  z^=z>>30; z*=0xBF58476D1CE4E5B9; z^=z>>27;
 *                                  z*=0x94D049BB133111EB; z^=z>>31
 *   mix32 is the 32-bit finaliser  x^=x>>16; x*=0x7FEB352D; x^=x>>15;
 *                                  x*=0x846CA68B; x^=x>>16
 *   G = 0x9E3779B97F4A7C15
 *   key(seed,step,chunk) = mix64( mix64(seed + G*(step+1)) + G*(chunk+1) )
 *   draw(key,j) = mix32( low32(key) + 0x9E3779B9*(j+1) ) ^ high32(key)
 *   bounded(d,b) = floor(d*b / 2^32)
 * All sums and products wrap modulo 2^64 (or 2^32 inside mix32/draw). */
static uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7FEB352Du;
    x ^= x >> 15;
    x *= 0x846CA68Bu;
    x ^= x >> 16;
    return x;
}

static uint64_t chunk_key(uint64_t seed, uint64_t step, uint64_t chunk)
{
    const uint64_t G = 0x9E3779B97F4A7C15ull;
    return mix64(mix64(seed + G * (step + 1)) + G * (chunk + 1));
}

static uint32_t draw(uint64_t key, uint32_t j)
{
    return mix32((uint32_t)key + 0x9E3779B9u * (j + 1u)) ^ (uint32_t)(key >> 32);
}

static int cmp_int32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* ------------------------------------------------------------ selection */

typedef struct {
    uint32_t mag; /* bit pattern of |c|: orders finite magnitudes, -0 == +0 */
    int32_t idx;
} orc_cand;

/* larger |c| first, then lower index */
static int cmp_cand(const void *a, const void *b)
{
    const orc_cand *x = (const orc_cand *)a, *y = (const orc_cand *)b;
    if (x->mag != y->mag) return (x->mag < y->mag) ? 1 : -1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

/* Indices kept in one chunk, ascending.  `chunk_id` is the chunk's global number
 * (it keys the Random scheme). */
static void select_chunk(const orc_config *cfg, const float *coeff, int64_t chunk_id,
                         int32_t *idx)
{
    const int s = cfg->chunk, k = cfg->topk;
    if (cfg->scheme == ORC_SCHEME_TOPK) {
        orc_cand cand[256];
        for (int j = 0; j < s; ++j) {
            float a = fabsf(coeff[j]);
            memcpy(&cand[j].mag, &a, 4);
            cand[j].idx = j;
        }
        qsort(cand, (size_t)s, sizeof(orc_cand), cmp_cand);
        for (int j = 0; j < k; ++j) idx[j] = cand[j].idx;
    } else if (cfg->scheme == ORC_SCHEME_STRIDE) {
        /* every n-th index, the offset rotating with the step */
        const int stride = s / k;
        const int off = (int)(cfg->step % (uint64_t)stride);
        for (int j = 0; j < k; ++j) idx[j] = off + j * stride;
    } else {
        /* k distinct indices: the first k places of a Fisher-Yates shuffle */
        int32_t perm[256];
        for (int j = 0; j < s; ++j) perm[j] = j;
        const uint64_t key = chunk_key(cfg->seed, cfg->step, (uint64_t)chunk_id);
        for (int j = 0; j < k; ++j) {
            uint32_t d = draw(key, (uint32_t)j);
            int t = j + (int)(((uint64_t)d * (uint64_t)(s - j)) >> 32);
            int32_t tmp = perm[j];
            perm[j] = perm[t];
            perm[t] = tmp;
        }
        for (int j = 0; j < k; ++j) idx[j] = perm[j];
    }
    qsort(idx, (size_t)k, sizeof(int32_t), cmp_int32);
}

/* idx[c*k + j] for chunks chunk0 .. chunk0+C-1; coeff is [C][s] (ignored by
 * Striding and Random, may be NULL for them). */
int orc_select(const orc_config *cfg, int64_t C, int64_t chunk0, const float *coeff,
               int32_t *idx)
{
    int rc = orc_check(cfg);
    if (rc) return rc;
    if (C > 0 && !idx) return ORC_ERR_NULL;
    if (C > 0 && cfg->scheme == ORC_SCHEME_TOPK && !coeff) return ORC_ERR_NULL;
    const int s = cfg->chunk, k = cfg->topk;
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < C; ++c)
        select_chunk(cfg, coeff ? coeff + c * s : NULL, chunk0 + c, idx + c * k);
    return ORC_OK;
}

/* ------------------------------------------- payload values and residual */

/* val[c*k+j] = coeff[c*s + idx[c*k+j]];
 * m_new[i] = fl32( m1[i] - sum_j D[idx_j][i - c*s] * val_j )      (m <- m - q)
 * In the identity domain q is the kept entries themselves, so they become 0. */
int orc_extract(const orc_config *cfg, int64_t n, const float *m1, const float *coeff,
                const int32_t *idx, float *val, float *m_new)
{
    int rc = orc_check(cfg);
    if (rc) return rc;
    if (n > 0 && (!m1 || !coeff || !idx || !val || !m_new)) return ORC_ERR_NULL;
    const int s = cfg->chunk, k = cfg->topk;
    const int64_t C = (n + s - 1) / s;
    const int use_dct = orc_uses_dct(cfg);
    double *D = NULL;
    if (use_dct) {
        D = (double *)malloc(sizeof(double) * s * s);
        orc_dct_matrix(s, D);
    }
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < C; ++c) {
        for (int j = 0; j < k; ++j) val[c * k + j] = coeff[c * s + idx[c * k + j]];
        for (int t = 0; t < s; ++t) {
            int64_t i = c * s + t;
            if (i >= n) break;
            double q = 0.0;
            for (int j = 0; j < k; ++j) {
                int32_t r = idx[c * k + j];
                double basis = use_dct ? D[(size_t)r * s + t] : (r == t ? 1.0 : 0.0);
                q += basis * (double)val[c * k + j];
            }
            m_new[i] = (float)((double)m1[i] - q);
        }
    }
    free(D);
    return ORC_OK;
}

/* Payload values in a 16-bit transfer dtype (val_bits), and the residual that removes from
 * the momentum exactly what the receivers will decode:
 * val_bits[c*k+j] = encode(coeff[c*s + idx]);  m_new = fl32( m1 - D^T decode(val_bits) ). */
int orc_extract_q(const orc_config *cfg, int64_t n, const float *m1, const float *coeff,
                  const int32_t *idx, int val_dtype, uint16_t *val_bits, float *m_new)
{
    int rc = orc_check(cfg);
    if (rc) return rc;
    if (val_dtype != ORC_BF16 && val_dtype != ORC_F16) return ORC_ERR_BAD_CONFIG;
    if (n > 0 && (!m1 || !coeff || !idx || !val_bits || !m_new)) return ORC_ERR_NULL;
    const int k = cfg->topk, s = cfg->chunk;
    const int64_t C = (n + s - 1) / s;
    float *decoded = (float *)malloc(sizeof(float) * (size_t)(C * k));
    float *shadow = (float *)malloc(sizeof(float) * (size_t)(C * s));
    memcpy(shadow, coeff, sizeof(float) * (size_t)(C * s));
    for (int64_t e = 0; e < C * k; ++e) {
        const int64_t at = (e / k) * s + idx[e];
        val_bits[e] = transfer_encode(val_dtype, coeff[at]);
        shadow[at] = transfer_decode(val_dtype, val_bits[e]);
    }
    /* orc_extract reads the kept values from the coefficient array it is given: hand it the
     * array with the kept entries replaced by their decoded transfer values */
    rc = orc_extract(cfg, n, m1, shadow, idx, decoded, m_new);
    free(shadow);
    free(decoded);
    return rc;
}

/* Averaged update before sign from payloads whose values are in a 16-bit transfer dtype. */
int orc_presign_q(const orc_config *cfg, int64_t n, int32_t R, const int32_t *idx,
                  int64_t idx_replica_stride, const uint16_t *val_bits, int val_dtype,
                  int64_t val_replica_stride, float *y)
{
    int rc = orc_check(cfg);
    if (rc) return rc;
    if (val_dtype != ORC_BF16 && val_dtype != ORC_F16) return ORC_ERR_BAD_CONFIG;
    if (R < 1) return ORC_ERR_BAD_CONFIG;
    if (n == 0) return ORC_OK;
    if (!val_bits || !y) return ORC_ERR_NULL;
    const int64_t entries = ((n + cfg->chunk - 1) / cfg->chunk) * cfg->topk;
    float *val = (float *)malloc(sizeof(float) * (size_t)(R * entries));
    for (int r = 0; r < R; ++r)
        for (int64_t e = 0; e < entries; ++e)
            val[r * entries + e] = transfer_decode(val_dtype, val_bits[r * val_replica_stride + e]);
    rc = orc_presign(cfg, n, R, idx, idx_replica_stride, val, entries, y);
    free(val);
    return rc;
}

/* ------------------------------------------------- ternary payload (sign before sync)
 * Discussion (the sign can be taken before the exchange, and a three-valued payload packs
 * more tightly) and Appendix B "Sign vs. No Sign": what travels is sign(c) in {-1, 0, +1}
 * of each kept coefficient (sign(0) = 0, as torch.sign).  Two bits per entry: 0 = zero,
 * 1 = +1, 3 = -1 (2 is never written and decodes to 0); 16 entries per 32-bit word, entry j
 * of chunk c in word c*W + j/16 at bits [2*(j%16), 2*(j%16)+2), W = ceil(k/16), so every chunk
 * starts on a word boundary.  The momentum loses the extracted components themselves
 * (Algorithm 1, "remove q from m"), whatever goes on the wire. */
int64_t orc_ternary_words(const orc_config *cfg, int64_t n)
{
    if (orc_check(cfg) || n < 0) return -1;
    return ((n + cfg->chunk - 1) / cfg->chunk) * ((cfg->topk + 15) / 16);
}

int orc_encode_ternary(const orc_config *cfg, int64_t n, const float *val, uint32_t *words)
{
    int rc = orc_check(cfg);
    if (rc) return rc;
    if (n > 0 && (!val || !words)) return ORC_ERR_NULL;
    const int k = cfg->topk, W = (k + 15) / 16;
    const int64_t C = (n + cfg->chunk - 1) / cfg->chunk;
    for (int64_t c = 0; c < C; ++c) {
        for (int w = 0; w < W; ++w) words[c * W + w] = 0u;
        for (int j = 0; j < k; ++j) {
            const float v = val[c * k + j];
            const uint32_t code = v > 0.0f ? 1u : (v < 0.0f ? 3u : 0u);
            words[c * W + j / 16] |= code << (2 * (j % 16));
        }
    }
    return ORC_OK;
}

int orc_decode_ternary(const orc_config *cfg, int64_t n, const uint32_t *words, float *val)
{
    int rc = orc_check(cfg);
    if (rc) return rc;
    if (n > 0 && (!val || !words)) return ORC_ERR_NULL;
    const int k = cfg->topk, W = (k + 15) / 16;
    const int64_t C = (n + cfg->chunk - 1) / cfg->chunk;
    for (int64_t c = 0; c < C; ++c)
        for (int j = 0; j < k; ++j) {
            const uint32_t code = (words[c * W + j / 16] >> (2 * (j % 16))) & 3u;
            val[c * k + j] = code == 1u ? 1.0f : (code == 3u ? -1.0f : 0.0f);
        }
    return ORC_OK;
}

/* Averaged update before sign from R ternary payloads (word_replica_stride in 32-bit words). */
int orc_presign_t(const orc_config *cfg, int64_t n, int32_t R, const int32_t *idx,
                  int64_t idx_replica_stride, const uint32_t *words, int64_t word_replica_stride,
                  float *y)
{
    int rc = orc_check(cfg);
    if (rc) return rc;
    if (R < 1) return ORC_ERR_BAD_CONFIG;
    if (n == 0) return ORC_OK;
    if (!words || !y) return ORC_ERR_NULL;
    const int64_t entries = ((n + cfg->chunk - 1) / cfg->chunk) * cfg->topk;
    float *val = (float *)malloc(sizeof(float) * (size_t)(R * entries));
    for (int r = 0; r < R && !rc; ++r)
        rc = orc_decode_ternary(cfg, n, words + r * word_replica_stride, val + r * entries);
    if (!rc) rc = orc_presign(cfg, n, R, idx, idx_replica_stride, val, entries, y);
    free(val);
    return rc;
}

/* The whole compress half: fold, transform, select, extract.
 * momentum is updated in place; idx_out may be NULL (Striding/Random callers do
 * not need it); coeff_out may be NULL. */
int orc_compress(const orc_config *cfg, int64_t n, const void *grad, int grad_dtype,
                 float *momentum, int32_t *idx_out, float *val_out, float *coeff_out)
{
    int rc = orc_check(cfg);
    if (rc) return rc;
    if (n == 0) return ORC_OK;
    if (!grad || !momentum || !val_out) return ORC_ERR_NULL;
    const int s = cfg->chunk, k = cfg->topk;
    const int64_t C = (n + s - 1) / s;
    float *m1 = (float *)malloc(sizeof(float) * (size_t)n);
    float *coeff = coeff_out ? coeff_out : (float *)malloc(sizeof(float) * (size_t)(C * s));
    int32_t *idx = idx_out ? idx_out : (int32_t *)malloc(sizeof(int32_t) * (size_t)(C * k));
    rc = orc_fold(cfg, n, grad, grad_dtype, momentum, m1);
    if (!rc) rc = orc_transform(cfg, n, m1, coeff);
    if (!rc) rc = orc_select(cfg, C, 0, coeff, idx);
    if (!rc) rc = orc_extract(cfg, n, m1, coeff, idx, val_out, momentum);
    if (!idx_out) free(idx);
    if (!coeff_out) free(coeff);
    free(m1);
    return rc;
}

/* ------------------------------------------------ decompress and update */

/* Synchronize: a[c][.] = (1/R) sum_r scatter(idx[r][c][.], val[r][c][.]).
 * idx may be NULL for Striding/Random: every replica used the same, regenerated
 * indices.  Duplicate indices add; indices outside [0,s) are ignored.
 * Then y = fl32(D^T a) (identity domain: y = fl32(a)); y is [n]. */
int orc_presign(const orc_config *cfg, int64_t n, int32_t R, const int32_t *idx,
                int64_t idx_replica_stride, const float *val, int64_t val_replica_stride,
                float *y)
{
    int rc = orc_check(cfg);
    if (rc) return rc;
    if (R < 1) return ORC_ERR_BAD_CONFIG;
    if (n == 0) return ORC_OK;
    if (!val || !y) return ORC_ERR_NULL;
    if (!idx && cfg->scheme == ORC_SCHEME_TOPK) return ORC_ERR_NULL;
    const int s = cfg->chunk, k = cfg->topk;
    const int64_t C = (n + s - 1) / s;
    const int use_dct = orc_uses_dct(cfg);
    double *D = NULL;
    if (use_dct) {
        D = (double *)malloc(sizeof(double) * s * s);
        orc_dct_matrix(s, D);
    }
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < C; ++c) {
        double a[256];
        int32_t own[256];
        for (int j = 0; j < s; ++j) a[j] = 0.0;
        if (!idx) select_chunk(cfg, NULL, c, own);
        for (int r = 0; r < R; ++r) {
            for (int j = 0; j < k; ++j) {
                int32_t p = idx ? idx[r * idx_replica_stride + c * k + j] : own[j];
                if (p < 0 || p >= s) continue;
                a[p] += (double)val[r * val_replica_stride + c * k + j];
            }
        }
        for (int j = 0; j < s; ++j) a[j] /= (double)R;
        for (int t = 0; t < s; ++t) {
            int64_t i = c * s + t;
            if (i >= n) break;
            double acc;
            if (use_dct) {
                acc = 0.0;
                for (int j = 0; j < s; ++j) acc += D[(size_t)j * s + t] * a[j];
            } else {
                acc = a[t];
            }
            y[i] = (float)acc;
        }
    }
    free(D);
    return ORC_OK;
}

/* Q = sign(y) if the sign flag is set (sign(0) = 0), else y;
 * theta <- round_to_dtype( theta*(1 - eta*lambda) - eta*Q ), in place. */
int orc_update(const orc_config *cfg, int64_t n, const float *y, void *params,
               int param_dtype)
{
    int rc = orc_check(cfg);
    if (rc) return rc;
    if (n > 0 && (!y || !params)) return ORC_ERR_NULL;
    const double eta = (double)cfg->lr, lambda = (double)cfg->weight_decay;
    const int use_sign = (cfg->flags & ORC_FLAG_SIGN) != 0;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double q = (double)y[i];
        if (use_sign) q = (q > 0.0) ? 1.0 : ((q < 0.0) ? -1.0 : 0.0);
        double th = load_elem(params, param_dtype, i);
        double nw = th * (1.0 - eta * lambda) - eta * q;
        if (param_dtype == ORC_BF16)
            ((uint16_t *)params)[i] = orc_double_to_bf16(nw);
        else
            ((float *)params)[i] = (float)nw;
    }
    return ORC_OK;
}

/* ------------------------------------------------- Decoupled AdamW variant */

/* Section "Decoupled AdamW": AdamW whose first and second moments (and, with amsgrad, the
 * running maximum of the second moment) stay local and are never synchronised; only Q is
 * shared.  The averaged update Q takes the place of the gradient in the textbook AdamW
 * step (Loshchilov & Hutter; Kingma & Ba), t counted from 1:
 *   m <- b1 m + (1-b1) Q,   v <- b2 v + (1-b2) Q^2,   vmax <- max(vmax, v)  (amsgrad)
 *   theta <- theta (1 - eta lambda) - eta/(1-b1^t) * m / ( sqrt(v or vmax)/sqrt(1-b2^t) + eps )
 * The moments are stored in fp32 and the stored values are the ones used for theta. */
typedef struct {
    float beta1;
    float beta2;
    float eps;
    int32_t amsgrad;
    uint64_t step;   /* t >= 1 */
} orc_adamw;

int orc_adamw_update(const orc_config *cfg, const orc_adamw *opt, int64_t n, const float *y,
                     void *params, int param_dtype, float *exp_avg, float *exp_avg_sq,
                     float *max_exp_avg_sq)
{
    int rc = orc_check(cfg);
    if (rc) return rc;
    if (!opt) return ORC_ERR_NULL;
    if (opt->step < 1) return ORC_ERR_BAD_CONFIG;
    if (n > 0 && (!y || !params || !exp_avg || !exp_avg_sq)) return ORC_ERR_NULL;
    if (n > 0 && opt->amsgrad && !max_exp_avg_sq) return ORC_ERR_NULL;
    const double eta = (double)cfg->lr, lambda = (double)cfg->weight_decay;
    const double b1 = (double)opt->beta1, b2 = (double)opt->beta2, eps = (double)opt->eps;
    const double bc1 = 1.0 - pow(b1, (double)opt->step);
    const double bc2 = 1.0 - pow(b2, (double)opt->step);
    const int use_sign = (cfg->flags & ORC_FLAG_SIGN) != 0;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double q = (double)y[i];
        if (use_sign) q = (q > 0.0) ? 1.0 : ((q < 0.0) ? -1.0 : 0.0);
        exp_avg[i] = (float)(b1 * (double)exp_avg[i] + (1.0 - b1) * q);
        exp_avg_sq[i] = (float)(b2 * (double)exp_avg_sq[i] + (1.0 - b2) * q * q);
        double vhat = (double)exp_avg_sq[i];
        if (opt->amsgrad) {
            if (vhat > (double)max_exp_avg_sq[i]) max_exp_avg_sq[i] = exp_avg_sq[i];
            vhat = (double)max_exp_avg_sq[i];
        }
        const double denom = sqrt(vhat) / sqrt(bc2) + eps;
        const double th = load_elem(params, param_dtype, i);
        const double nw = th * (1.0 - eta * lambda) - (eta / bc1) * (double)exp_avg[i] / denom;
        if (param_dtype == ORC_BF16)
            ((uint16_t *)params)[i] = orc_double_to_bf16(nw);
        else
            ((float *)params)[i] = (float)nw;
    }
    return ORC_OK;
}

/* The whole decompress half.  presign_out may be NULL. */
int orc_decompress_step(const orc_config *cfg, int64_t n, int32_t R, const int32_t *idx,
                        int64_t idx_replica_stride, const float *val,
                        int64_t val_replica_stride, void *params, int param_dtype,
                        float *presign_out)
{
    int rc = orc_check(cfg);
    if (rc) return rc;
    if (n == 0) return ORC_OK;
    float *y = presign_out ? presign_out : (float *)malloc(sizeof(float) * (size_t)n);
    rc = orc_presign(cfg, n, R, idx, idx_replica_stride, val, val_replica_stride, y);
    if (!rc) rc = orc_update(cfg, n, y, params, param_dtype);
    if (!presign_out) free(y);
    return rc;
}
