/*
 * detonation.h — C ABI of the MI355X (gfx950) library for the per-step optimizer
 * hot path of FlexDeMo / DeMo-SGD (arXiv 2502.06728, Algorithm 1) on one GPU's
 * flat FSDP shard.
 *
 * The step has two halves with the inter-node exchange between them:
 *
 *   detonation_compress          m <- beta*m + g;  q <- ExtractFastComponents(m,s,k);
 *                                m <- m - q;  emit q as a sparse payload
 *   (all_gather of payloads over the replication group R — not part of this library)
 *   detonation_decompress_step   Q <- mean of R payloads, back in parameter space,
 *                                optional sign;  theta <- theta*(1-eta*lambda) - eta*Q
 *
 * Notation: n = shard length, s = chunk size, k = TopK, C = ceil(n/s) chunks.  The
 * shard is cut into chunks of s consecutive elements, ignoring tensor boundaries;
 * the last chunk is zero-extended and its pad positions are never written.  The
 * transform is the orthonormal DCT-II  D[j][i] = a_j cos(pi (2i+1) j / (2s)),
 * a_0 = sqrt(1/s), a_j = sqrt(2/s); its inverse is its transpose.
 *
 * Common rules for every entry point
 *   - All data pointers are DEVICE pointers on the current HIP device.  `cfg` is a
 *     HOST pointer, read before the call returns.
 *   - The caller owns every buffer and keeps it alive until `stream` has run the
 *     call.  The library allocates nothing, keeps no state between calls and never
 *     synchronises: work is enqueued on `stream` (a hipStream_t; NULL = the default
 *     stream) and the call returns.
 *   - The return value is a deto_status.  Host-side arguments are validated; device
 *     data is not (an out-of-range payload index is skipped, not reported).
 *   - Buffers must not overlap each other.
 *   - DETO_ERR_HIP reports the launches of this call only: a call that gets as far as
 *     launching first resets the HIP runtime's sticky last-error state (hipGetLastError), so
 *     an error left by an earlier, unrelated HIP call is neither reported here nor left behind.
 *   - Alignment.  Every pointer must be aligned to its element size (else DETO_ERR_ALIGN).
 *     The bandwidth kernels additionally need 16-byte aligned grad, momentum, params, optimizer
 *     state and debug arrays, and payload arrays aligned to one lane's access: when k is a
 *     multiple of 4, four consecutive entries (16 bytes of fp32 values or int32 indices,
 *     8 bytes of 16-bit values, 4 bytes of byte indices; 8 bytes of two-bit signs when k > 16,
 *     else 4), otherwise one element.  This holds for the base of idx / val and for every
 *     replica offset r*stride, so the contiguous [R][C*k] buffer an all_gather returns always
 *     qualifies for fp32 + int32 payloads.  Buffers that do not meet this are still processed
 *     correctly, by general kernels that are more than ten times slower.
 *   - Environment.  DETO_SMALL_SHARD_TILES (a count of 64-chunk tiles, default 8192; read at
 *     every call) is the shard size up to which the compress half at chunk size 64 and 128
 *     (top-k, fp32 + int32 payload) spreads a tile over more wavefronts: shorter launches on
 *     small shards, a few per cent longer ones on large shards.  0 switches it off.  The
 *     results of the two kernel choices agree to rounding.
 */
#ifndef DETONATION_H
#define DETONATION_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DETO_OK = 0,
    DETO_ERR_NULL = 1,         /* a required pointer is NULL */
    DETO_ERR_BAD_CONFIG = 2,   /* chunk/topk/scheme/dtype/R/n/stride out of range */
    DETO_ERR_UNSUPPORTED = 3,  /* meaningful request outside what this build covers: a
                                  replication group of more than 64 replicas */
    DETO_ERR_ALIGN = 4,        /* a pointer is not aligned to its element size */
    DETO_ERR_HIP = 5           /* the HIP runtime refused the launch */
} deto_status;

/* Replication scheme (paper, "Replication Schemes").
 *   TOPK   : DeMo — the k largest-magnitude DCT coefficients of each chunk; ties go
 *            to the lower index.  Indices are part of the payload.
 *   STRIDE : every (s/k)-th position of each chunk, indices o + j*floor(s/k),
 *            o = step mod floor(s/k).  Indices are not transmitted.
 *   RANDOM : k distinct positions per chunk, the first k places of a Fisher-Yates
 *            shuffle driven by a counter-based generator keyed (seed, step, chunk),
 *            so every replica regenerates them.  Indices are not transmitted. */
typedef enum { DETO_SCHEME_TOPK = 0, DETO_SCHEME_STRIDE = 1, DETO_SCHEME_RANDOM = 2 } deto_scheme;

/* Element types.  Gradients and parameters are F32 or BF16; payload values may also be F16
 * (IEEE half) or TERNARY (only the sign, two bits per entry; see detonation_compress_packed). */
typedef enum { DETO_F32 = 0, DETO_BF16 = 1, DETO_F16 = 2, DETO_TERNARY = 3 } deto_dtype;

/* Payload index width: chunk-local indices always fit a byte (s <= 256). */
typedef enum { DETO_IDX_I32 = 0, DETO_IDX_U8 = 1 } deto_idx_dtype;

enum {
    DETO_FLAG_SIGN = 1u, /* apply sign() (sign(0)=0) to the averaged update before the
                            parameter step (paper, "Overall Setup", Appendix B) */
    DETO_FLAG_DCT = 2u   /* STRIDE/RANDOM pick DCT coefficients instead of raw momentum
                            entries.  TOPK always works on coefficients. */
};

typedef struct {
    int32_t chunk;        /* s, 1..256 (the paper sweeps 16..256, Appendix B) */
    int32_t topk;         /* k, 1..s; compression rate = k/s */
    int32_t scheme;       /* deto_scheme */
    uint32_t flags;       /* DETO_FLAG_* */
    float decay;          /* beta, Algorithm 1 */
    float lr;             /* eta, Algorithm 1 */
    float weight_decay;   /* lambda, decoupled: theta*(1 - eta*lambda) */
    uint64_t seed;        /* RANDOM: shared by all replicas */
    uint64_t step;        /* optimizer step: STRIDE offset, RANDOM stream */
} deto_config;

/*
 * Compress half (Algorithm 1: accumulate, ExtractFastComponents, remove q from m).
 *
 *   m1 = beta*momentum + grad                       (fp32)
 *   c  = D * m1 per chunk           (or c = m1 for STRIDE/RANDOM without DETO_FLAG_DCT)
 *   I  = the k indices the scheme keeps in each chunk, ascending
 *   val_out[ch*k + j] = c[ch][I_j],  idx_out[ch*k + j] = I_j   (chunk-local, 0..s-1)
 *   momentum = m1 - D^T * (c restricted to I)       (in place)
 *
 *   grad        device, [n] of grad_dtype (deto_dtype), read only
 *   momentum    device, [n] fp32, in: m_t, out: m_{t+1}
 *   idx_out     device, [C*k] int32; may be NULL for STRIDE/RANDOM
 *   val_out     device, [C*k] fp32
 *   coeff_dbg   device, [C*s] fp32 or NULL: receives c (zero-extended last chunk).
 *               For parity checks only; leave NULL when timing.
 *
 * Errors: DETO_ERR_NULL (cfg, grad, momentum, val_out, or idx_out for TOPK, is NULL
 * while n > 0), DETO_ERR_BAD_CONFIG, DETO_ERR_ALIGN, DETO_ERR_HIP.  n = 0 is a no-op.
 */
int detonation_compress(const deto_config* cfg, int64_t n,
                        const void* grad, int grad_dtype,
                        float* momentum,
                        int32_t* idx_out, float* val_out,
                        float* coeff_dbg,
                        void* stream);

/*
 * Decompress-and-update half (Algorithm 1: Synchronize result -> parameter update).
 *
 *   a[ch][i] = (1/R) * sum_r sum_j [idx[r][ch][j] == i] * val[r][ch][j]
 *   y  = D^T * a per chunk          (or y = a without the DCT domain)
 *   Q  = sign(y) if DETO_FLAG_SIGN else y
 *   params = round_to_dtype( params*(1 - eta*lambda) - eta*Q )   (in place)
 *
 *   R           number of replica payloads, 1..64.  64 is the largest replication group the
 *               paper runs (section "OLMo2: Scaling Up", 64 nodes) and the largest this
 *               library is tested with; R > 64 returns DETO_ERR_UNSUPPORTED, R < 1
 *               DETO_ERR_BAD_CONFIG.
 *   idx         device, replica r at idx + r*idx_replica_stride, each [C*k] int32 as an
 *               all_gather leaves them; NULL for STRIDE/RANDOM (indices regenerated from
 *               cfg, identical for every replica).  Duplicate indices add; indices
 *               outside [0,s) are skipped.
 *   val         device, replica r at val + r*val_replica_stride, each [C*k] fp32
 *   strides     in elements, >= C*k (ignored when R == 1); see "Alignment" above for the
 *               multiples that keep the bandwidth kernels in use
 *   params      device, [n] of param_dtype, updated in place (bf16: round to nearest even)
 *   presign_dbg device, [n] fp32 or NULL: receives y.  Parity checks only.
 *
 * Errors as for detonation_compress.  n = 0 is a no-op.
 */
int detonation_decompress_step(const deto_config* cfg, int64_t n, int32_t R,
                               const int32_t* idx, int64_t idx_replica_stride,
                               const float* val, int64_t val_replica_stride,
                               void* params, int param_dtype,
                               float* presign_dbg,
                               void* stream);

/*
 * The same two halves with a narrower payload (paper, Appendix B "Communication Floating Point
 * Data Type": values sent as fp16 instead of fp32; "Replicator bandwidth usage": the indices
 * are half of DeMo's traffic).  Values travel as val_dtype (DETO_F32, DETO_BF16 or DETO_F16,
 * rounded to nearest even), indices as idx_dtype (DETO_IDX_I32 or DETO_IDX_U8).  The
 * momentum gives up exactly what the receivers will decode:
 *     momentum = m1 - D^T * decode(encode(c restricted to I)),
 * so the rounding error of the transfer stays in the local momentum.  Everything else, the
 * argument rules and the error codes are those of detonation_compress and
 * detonation_decompress_step, which are these calls with DETO_IDX_I32 and DETO_F32; replica
 * strides are in elements of the respective dtype.
 *
 * DETO_TERNARY is the variant in which the sign is taken before the exchange (paper,
 * Discussion; Appendix B "Sign vs. No Sign"): only sign(c) in {-1, 0, +1} of each kept coefficient travels (sign(0) = 0).  Two
 * bits per entry (0 = zero, 1 = +1, 3 = -1; 2 is never written and decodes to 0), 16 entries
 * per uint32 word, entry j of chunk ch in word ch*W + j/16 at bits [2*(j%16), 2*(j%16)+2),
 * W = ceil(k/16): every chunk starts on a word boundary and val_out / val hold
 * detonation_ternary_words(cfg, n) = C*W words per replica (replica stride in words, pointers
 * 4-byte aligned).  The momentum gives up the extracted components themselves (Algorithm 1,
 * "remove q from m"), as with DETO_F32.  The receivers average the signs of the R replicas,
 * transform back and, with DETO_FLAG_SIGN, take the sign of the result once more.
 */
int detonation_compress_packed(const deto_config* cfg, int64_t n,
                               const void* grad, int grad_dtype,
                               float* momentum,
                               void* idx_out, int idx_dtype,
                               void* val_out, int val_dtype,
                               float* coeff_dbg,
                               void* stream);

int detonation_decompress_step_packed(const deto_config* cfg, int64_t n, int32_t R,
                                      const void* idx, int idx_dtype, int64_t idx_replica_stride,
                                      const void* val, int val_dtype, int64_t val_replica_stride,
                                      void* params, int param_dtype,
                                      float* presign_dbg,
                                      void* stream);

/* Decoupled AdamW (paper, section "Decoupled AdamW"): AdamW whose first and second moments
 * (and, with amsgrad, the running maximum of the second moment) are local to the rank and
 * never synchronised.  The averaged update Q takes the place of the gradient:
 *   m <- b1 m + (1-b1) Q,  v <- b2 v + (1-b2) Q^2,  vmax <- max(vmax, v)   (amsgrad)
 *   params <- params (1 - eta lambda) - eta/(1-b1^t) * m / ( sqrt(v or vmax)/sqrt(1-b2^t) + eps ) */
typedef struct {
    float beta1;
    float beta2;
    float eps;
    int32_t amsgrad;   /* 0 or 1 */
    uint64_t step;     /* t, counted from 1 (bias correction) */
} deto_adamw;

/*
 * detonation_decompress_step with Decoupled AdamW as the underlying optimizer: Q is computed
 * exactly as there (scatter R payloads, average, inverse DCT, optional sign) and then drives
 * the AdamW step above instead of the plain SGD update.
 *
 *   exp_avg, exp_avg_sq   device, [n] fp32, updated in place
 *   max_exp_avg_sq        device, [n] fp32, updated in place; required iff opt->amsgrad
 *   everything else       as for detonation_decompress_step (fp32 values, int32 indices)
 *
 * Errors as there, plus DETO_ERR_NULL for a missing state array and DETO_ERR_BAD_CONFIG for
 * opt->step == 0 or betas outside [0,1).
 */
int detonation_decompress_adamw_step(const deto_config* cfg, const deto_adamw* opt, int64_t n,
                                     int32_t R,
                                     const int32_t* idx, int64_t idx_replica_stride,
                                     const float* val, int64_t val_replica_stride,
                                     void* params, int param_dtype,
                                     float* exp_avg, float* exp_avg_sq, float* max_exp_avg_sq,
                                     float* presign_dbg,
                                     void* stream);

/*
 * detonation_decompress_adamw_step for payloads in the formats of
 * detonation_decompress_step_packed (paper, "Overall Setup": the experiments synchronise only
 * the signs, and Decoupled AdamW is one of the underlying optimizers they run on top of that;
 * Appendix B, "Communication Floating Point Data Type" for the 16-bit formats).  idx / val,
 * their dtypes and replica strides as for detonation_decompress_step_packed; the optimizer
 * state and all errors as for detonation_decompress_adamw_step.
 */
int detonation_decompress_adamw_step_packed(const deto_config* cfg, const deto_adamw* opt,
                                            int64_t n, int32_t R,
                                            const void* idx, int idx_dtype,
                                            int64_t idx_replica_stride,
                                            const void* val, int val_dtype,
                                            int64_t val_replica_stride,
                                            void* params, int param_dtype,
                                            float* exp_avg, float* exp_avg_sq,
                                            float* max_exp_avg_sq,
                                            float* presign_dbg,
                                            void* stream);

/*
 * The first line of Algorithm 1 alone: momentum <- beta*momentum + grad, nothing extracted and
 * nothing sent.  For replicators that do not exchange on every step (paper, "Replication
 * Schemes": DiLoCo, which synchronises only on every n-th optimizer step): the steps in between
 * accumulate with this call; the synchronising step is detonation_compress with
 * DETO_SCHEME_STRIDE and topk = chunk (every position is taken, so the whole momentum is the
 * payload and restarts from zero) followed by detonation_decompress_step.
 *
 *   grad        device, [n] of grad_dtype, read only
 *   momentum    device, [n] fp32, updated in place
 *
 * Only cfg->decay is used, but cfg is validated as a whole.  Errors: DETO_ERR_NULL,
 * DETO_ERR_BAD_CONFIG, DETO_ERR_ALIGN, DETO_ERR_HIP.  n = 0 is a no-op.
 */
int detonation_accumulate(const deto_config* cfg, int64_t n,
                          const void* grad, int grad_dtype,
                          float* momentum,
                          void* stream);

/* Payload entries per replica, ceil(n/s)*k (the paper's compression rate k/s times the
 * padded shard length); -1 if cfg is invalid. */
int64_t detonation_payload_entries(const deto_config* cfg, int64_t n);

/* 32-bit words of one replica's DETO_TERNARY payload, ceil(n/s)*ceil(k/16); -1 if cfg is
 * invalid. */
int64_t detonation_ternary_words(const deto_config* cfg, int64_t n);

/* Static, human-readable name of a deto_status. */
const char* detonation_status_string(int status);

/* ABI version of this header: major*1000 + minor (1001: the *_packed entry points; 1002: Decoupled AdamW; 1003: DETO_TERNARY; 1004: detonation_accumulate; 1005: detonation_decompress_adamw_step_packed; 1006: R > 64 is DETO_ERR_UNSUPPORTED, payload alignment by lane access, last-error reset; 1007: kernel choice by shard size, DETO_SMALL_SHARD_TILES). */
int detonation_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DETONATION_H */
