// C ABI of the library (see include/detonation.h): argument validation, resolution of
// deto_config into kernel parameters, kernel selection and launch.  Nothing is allocated and
// no tensor data is touched on the host; every call only enqueues kernels on the caller's
// stream.  What the host does compute are kernel parameters derived from deto_config: the
// scale factors of the transform, the bias corrections of AdamW, and Striding's kept positions
// (an integer pattern that is the same for every chunk: stride_pattern, stride_geom), which
// the kernels take by value.
#include "../../include/detonation.h"

#include <hip/hip_runtime.h>

#include <cmath>

#include "deto_device.hip.h"
#include "generic_kernels.hip.h"
#include "tiled_launch.h"

namespace {

using deto::KParams;

int validate(const deto_config* cfg) {
    if (!cfg) return DETO_ERR_NULL;
    if (cfg->chunk < 1 || cfg->chunk > deto::kMaxChunk) return DETO_ERR_BAD_CONFIG;
    if (cfg->topk < 1 || cfg->topk > cfg->chunk) return DETO_ERR_BAD_CONFIG;
    if (cfg->scheme < DETO_SCHEME_TOPK || cfg->scheme > DETO_SCHEME_RANDOM)
        return DETO_ERR_BAD_CONFIG;
    if (cfg->flags & ~(DETO_FLAG_SIGN | DETO_FLAG_DCT)) return DETO_ERR_BAD_CONFIG;
    if (!std::isfinite(cfg->decay) || !std::isfinite(cfg->lr) || !std::isfinite(cfg->weight_decay))
        return DETO_ERR_BAD_CONFIG;
    return DETO_OK;
}

bool valid_dtype(int d) { return d == DETO_F32 || d == DETO_BF16; }

bool valid_val_dtype(int d) {
    return d == DETO_F32 || d == DETO_BF16 || d == DETO_F16 || d == DETO_TERNARY;
}

bool valid_idx_dtype(int d) { return d == DETO_IDX_I32 || d == DETO_IDX_U8; }

size_t idx_size(int d) { return d == DETO_IDX_U8 ? 1 : 4; }

size_t val_size(int d) { return (d == DETO_F32 || d == DETO_TERNARY) ? 4 : 2; }

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

size_t elem_size(int dtype) { return dtype == DETO_BF16 ? 2 : 4; }

KParams resolve(const deto_config* cfg, int R, int val_dtype, int idx_dtype) {
    KParams p = {};
    p.val_dtype = val_dtype;
    p.idx_u8 = idx_dtype == DETO_IDX_U8 ? 1 : 0;
    p.s = cfg->chunk;
    p.k = cfg->topk;
    p.scheme = cfg->scheme;
    p.use_dct = (cfg->scheme == DETO_SCHEME_TOPK || (cfg->flags & DETO_FLAG_DCT)) ? 1 : 0;
    p.use_sign = (cfg->flags & DETO_FLAG_SIGN) ? 1 : 0;
    p.R = R;
    p.beta = cfg->decay;
    p.lr = cfg->lr;
    p.wd_scale = static_cast<float>(1.0 - static_cast<double>(cfg->lr) *
                                              static_cast<double>(cfg->weight_decay));
    p.alpha0 = static_cast<float>(std::sqrt(1.0 / cfg->chunk));
    p.alpha = static_cast<float>(std::sqrt(2.0 / cfg->chunk));
    p.inv_R = static_cast<float>(1.0 / R);
    p.seed = cfg->seed;
    p.step = cfg->step;
    return p;
}

int64_t chunks_of(int64_t n, int s) { return (n + s - 1) / s; }

unsigned grid_for(int64_t chunks) {
    const int64_t cap = 256 * 32;  // 256 CUs, several single-wave workgroups each
    return static_cast<unsigned>(chunks < cap ? chunks : cap);
}

// Status of the launches of this call.  Every compute entry point calls fresh_status() before
// its first launch, so an error left behind by an earlier, unrelated HIP call of the process is
// not reported as this call's.
void fresh_status() { (void)hipGetLastError(); }
int launched() { return hipGetLastError() == hipSuccess ? DETO_OK : DETO_ERR_HIP; }

// grid of a grid-stride streaming kernel (256 lanes per workgroup) over `items` lane-items:
// one item per lane.  Many short-lived workgroups stream faster on this GPU than a few
// thousand looping ones (plain copy: 6.2 TB/s with 262,144 workgroups, 4.8 TB/s with 2,048).
unsigned stream_grid(int64_t items) {
    const int64_t want = (items + 255) / 256 + 1;
    return static_cast<unsigned>(want < 0x7FFFFFFF ? want : 0x7FFFFFFF);
}

bool aligned16(const void* p) { return aligned(p, 16); }

// Width in bytes of one lane's access to a payload array in the lane-per-chunk, two-lane and
// matrix-core kernels: four consecutive entries when k is a multiple of 4 (16 bytes of fp32 or
// int32, 8 bytes of 16-bit values, 4 bytes of byte indices; a chunk's one or two words of two-bit
// signs), a single element otherwise.  The array's base and every replica's offset from it
// must be multiples of this for those kernels to be used.
size_t idx_access(const KParams& p) {
    if (p.k % 4 != 0) return p.idx_u8 ? 1 : 4;
    return p.idx_u8 ? 4 : 16;
}
size_t val_access(const KParams& p) {
    if (p.val_dtype == DETO_TERNARY) return p.k > 16 ? 8 : 4;
    if (p.k % 4 != 0) return val_size(p.val_dtype);
    return p.val_dtype == DETO_F32 ? 16 : 8;
}

// tiled kernels take one 64-chunk tile per workgroup
constexpr int64_t kMaxTiles = 0x7FFFFFFF;

// Striding: the positions o + j*floor(s/k) as a bit pattern (chunk sizes up to 128)
void stride_pattern(const KParams& p, uint32_t (&w)[4]) {
    w[0] = w[1] = w[2] = w[3] = 0u;
    if (p.s > 128) return;
    const int stride = p.s / p.k;
    const int off = static_cast<int>(p.step % static_cast<uint64_t>(stride));
    for (int j = 0; j < p.k; ++j) {
        const int at = off + j * stride;
        w[at / 32] |= 1u << (at % 32);
    }
}

}  // namespace

extern "C" {

int detonation_compress_packed(const deto_config* cfg, int64_t n, const void* grad,
                               int grad_dtype, float* momentum, void* idx_out, int idx_dtype,
                               void* val_out, int val_dtype, float* coeff_dbg, void* stream) {
    int rc = validate(cfg);
    if (rc) return rc;
    if (n < 0 || !valid_dtype(grad_dtype) || !valid_val_dtype(val_dtype) ||
        !valid_idx_dtype(idx_dtype))
        return DETO_ERR_BAD_CONFIG;
    if (n == 0) return DETO_OK;
    if (!grad || !momentum || !val_out) return DETO_ERR_NULL;
    if (cfg->scheme == DETO_SCHEME_TOPK && !idx_out) return DETO_ERR_NULL;
    if (!aligned(grad, elem_size(grad_dtype)) || !aligned(momentum, 4) ||
        !aligned(val_out, val_size(val_dtype)) || !aligned(idx_out, idx_size(idx_dtype)) ||
        !aligned(coeff_dbg, 4))
        return DETO_ERR_ALIGN;

    const KParams p = resolve(cfg, 1, val_dtype, idx_dtype);
    const int64_t C = chunks_of(n, p.s);
    hipStream_t st = static_cast<hipStream_t>(stream);
    fresh_status();

    // every position kept in the raw domain: the payload is the folded momentum itself
    if (p.scheme != DETO_SCHEME_TOPK && !p.use_dct && p.k == p.s && val_dtype == DETO_F32 &&
        idx_dtype == DETO_IDX_I32) {
        const bool vec = p.s % 4 == 0 && aligned16(grad) && aligned16(momentum) &&
                         aligned16(idx_out) && aligned16(val_out) && aligned16(coeff_dbg);
        const unsigned grid = stream_grid(C * p.s / 4);
        int32_t* io = static_cast<int32_t*>(idx_out);
        float* vo = static_cast<float*>(val_out);
        const int64_t entries = C * p.s;
        if (grad_dtype == DETO_BF16) {
            if (vec) deto::compress_dense_kernel<true, true><<<grid, 256, 0, st>>>(
                         p, n, entries, grad, momentum, io, vo, coeff_dbg);
            else deto::compress_dense_kernel<true, false><<<grid, 256, 0, st>>>(
                         p, n, entries, grad, momentum, io, vo, coeff_dbg);
        } else {
            if (vec) deto::compress_dense_kernel<false, true><<<grid, 256, 0, st>>>(
                         p, n, entries, grad, momentum, io, vo, coeff_dbg);
            else deto::compress_dense_kernel<false, false><<<grid, 256, 0, st>>>(
                         p, n, entries, grad, momentum, io, vo, coeff_dbg);
        }
        return launched();
    }

    // a tiled kernel if one exists (full 64-chunk tiles plus, in the same launch, the tail
    // chunks on the general code), else the general kernel for everything
    int64_t c0 = 0;
    const int64_t tiles = (n / p.s) / deto::kWave;
    if (tiles <= kMaxTiles && aligned16(grad) && aligned16(momentum) &&
        aligned(idx_out, idx_access(p)) && aligned(val_out, val_access(p)) &&
        aligned16(coeff_dbg)) {
        deto::CompressLaunch a{p, tiles, n, C, grad, grad_dtype == DETO_BF16, momentum, idx_out,
                               val_out, coeff_dbg, {0, 0, 0, 0}, st};
        stride_pattern(p, a.stride_mask);
        // (chunk 64 on a small shard: two wavefronts per tile, see small_shard_tiles)
        const bool done = tiles == 0 ? false
                          : (p.scheme == DETO_SCHEME_TOPK)
                              ? (deto::launch_compress_split_64(a) > 0 ||
                                 deto::launch_compress_topk_s64(a) ||
                                 deto::launch_compress_topk_s32(a) ||
                                 deto::launch_compress_topk_s16(a) ||
                                 deto::launch_compress_topk_packed(a) ||
                                 deto::launch_compress_topk_packed_s32(a) ||
                                 deto::launch_compress_topk_ternary(a))
                              : (deto::launch_compress_scheme(a) ||
                                 deto::launch_compress_scheme_small(a) ||
                                 deto::launch_compress_scheme_narrow_s32(a) ||
                                 deto::launch_compress_scheme_narrow_s64(a));
        if (done) {
            rc = launched();
            if (rc) return rc;
            c0 = C;   // the tail chunks rode along in the same launch
        } else {
            // no lane-per-chunk kernel for this (s, k): chunk 96, 128, 192 and 256 run with a
            // wavefront per coefficient class (fp32 + int32 payloads, k <= s/2) or two lanes
            // per chunk (other formats), anything else on the matrix-core kernel, which takes
            // the leading multiple of 32 chunks
            c0 = deto::launch_compress_split(a);
            if (c0 == 0) c0 = deto::launch_compress_pair(a);
            if (c0 == 0) c0 = deto::launch_compress_mfma(a);
            if (c0 > 0) {
                rc = launched();
                if (rc) return rc;
            }
        }
    }
    // Striding in the raw domain at a shape without a lane-per-chunk kernel: it does not look
    // at the values, so a plain streaming kernel serves any chunk size and k
    if (c0 == 0 && p.scheme == DETO_SCHEME_STRIDE && !p.use_dct && val_dtype == DETO_F32 &&
        idx_dtype == DETO_IDX_I32) {
        const deto::StrideGeom sg = deto::stride_geom(p.s, p.k, p.step);
        const int64_t padded = C * p.s;
        const int64_t wgs = (padded + deto::kStrideSpan - 1) / deto::kStrideSpan;
        if (wgs <= 0x7FFFFFFF) {
            const unsigned grid = static_cast<unsigned>(wgs);
            if (grad_dtype == DETO_BF16)
                deto::compress_stride_kernel<true><<<grid, 256, 0, st>>>(
                    p, n, padded, sg, grad, momentum, static_cast<int32_t*>(idx_out),
                    static_cast<float*>(val_out), coeff_dbg);
            else
                deto::compress_stride_kernel<false><<<grid, 256, 0, st>>>(
                    p, n, padded, sg, grad, momentum, static_cast<int32_t*>(idx_out),
                    static_cast<float*>(val_out), coeff_dbg);
            return launched();
        }
    }
    if (c0 < C) {
        const unsigned grid = grid_for(C - c0);
        if (grad_dtype == DETO_BF16)
            deto::compress_generic<true><<<grid, deto::kWave, 0, st>>>(
                p, n, c0, C, grad, momentum, idx_out, val_out, coeff_dbg);
        else
            deto::compress_generic<false><<<grid, deto::kWave, 0, st>>>(
                p, n, c0, C, grad, momentum, idx_out, val_out, coeff_dbg);
        rc = launched();
    }
    return rc;
}

int detonation_compress(const deto_config* cfg, int64_t n, const void* grad, int grad_dtype,
                        float* momentum, int32_t* idx_out, float* val_out, float* coeff_dbg,
                        void* stream) {
    return detonation_compress_packed(cfg, n, grad, grad_dtype, momentum, idx_out, DETO_IDX_I32,
                                      val_out, DETO_F32, coeff_dbg, stream);
}

}  // extern "C"

namespace {

// Both decompress entry points: `opt` is null for the plain SGD update.
int decompress_impl(const deto_config* cfg, const deto_adamw* opt, int64_t n, int32_t R,
                    const void* idx, int idx_dtype, int64_t idx_replica_stride, const void* val,
                    int val_dtype, int64_t val_replica_stride, void* params, int param_dtype,
                    deto::AdamPtrs adam, float* presign_dbg, void* stream) {
    int rc = validate(cfg);
    if (rc) return rc;
    if (opt) {
        if (opt->step < 1 || !(opt->beta1 >= 0.0f && opt->beta1 < 1.0f) ||
            !(opt->beta2 >= 0.0f && opt->beta2 < 1.0f) || !std::isfinite(opt->eps) ||
            (opt->amsgrad != 0 && opt->amsgrad != 1))
            return DETO_ERR_BAD_CONFIG;
    }
    if (n < 0 || !valid_dtype(param_dtype) || R < 1 || !valid_val_dtype(val_dtype) ||
        !valid_idx_dtype(idx_dtype))
        return DETO_ERR_BAD_CONFIG;
    // the largest replication group of the paper (and of this library's tests)
    if (R > deto::kMaxReplicas) return DETO_ERR_UNSUPPORTED;
    if (n == 0) return DETO_OK;
    if (!val || !params) return DETO_ERR_NULL;
    if (cfg->scheme == DETO_SCHEME_TOPK && !idx) return DETO_ERR_NULL;
    if (opt && (!adam.m || !adam.v || (opt->amsgrad && !adam.vmax))) return DETO_ERR_NULL;
    if (!aligned(params, elem_size(param_dtype)) || !aligned(val, val_size(val_dtype)) ||
        !aligned(idx, idx_size(idx_dtype)) || !aligned(presign_dbg, 4) || !aligned(adam.m, 4) ||
        !aligned(adam.v, 4) || !aligned(adam.vmax, 4))
        return DETO_ERR_ALIGN;

    KParams p = resolve(cfg, R, val_dtype, idx_dtype);
    if (opt) {
        const double bc1 = 1.0 - std::pow(static_cast<double>(opt->beta1),
                                          static_cast<double>(opt->step));
        const double bc2 = 1.0 - std::pow(static_cast<double>(opt->beta2),
                                          static_cast<double>(opt->step));
        p.adam = 1;
        p.amsgrad = opt->amsgrad;
        p.b1 = opt->beta1;
        p.b2 = opt->beta2;
        p.omb1 = static_cast<float>(1.0 - static_cast<double>(opt->beta1));
        p.omb2 = static_cast<float>(1.0 - static_cast<double>(opt->beta2));
        p.eps = opt->eps;
        p.step_size = static_cast<float>(static_cast<double>(cfg->lr) / bc1);
        p.inv_sqrt_bc2 = static_cast<float>(1.0 / std::sqrt(bc2));
    }
    const int64_t C = chunks_of(n, p.s);
    const int64_t entries = C * p.k;
    // a replica's values: one element per entry, or ceil(k/16) words per chunk (ternary)
    const int64_t val_elems = val_dtype == DETO_TERNARY ? C * ((p.k + 15) / 16) : entries;
    if (R > 1 && (val_replica_stride < val_elems || (idx && idx_replica_stride < entries)))
        return DETO_ERR_BAD_CONFIG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    fresh_status();

    // every position kept in the raw domain: the mean of R dense arrays drives the update
    if (!idx && !opt && !p.use_dct && p.k == p.s && val_dtype == DETO_F32) {
        const bool vec = aligned16(val) && aligned16(params) && aligned16(presign_dbg) &&
                         (R == 1 || val_replica_stride % 4 == 0);
        const unsigned grid = stream_grid(n / 4);
        const float* v = static_cast<const float*>(val);
        if (param_dtype == DETO_BF16) {
            if (vec) deto::decompress_dense_kernel<true, true><<<grid, 256, 0, st>>>(
                         p, n, v, val_replica_stride, params, presign_dbg);
            else deto::decompress_dense_kernel<true, false><<<grid, 256, 0, st>>>(
                         p, n, v, val_replica_stride, params, presign_dbg);
        } else {
            if (vec) deto::decompress_dense_kernel<false, true><<<grid, 256, 0, st>>>(
                         p, n, v, val_replica_stride, params, presign_dbg);
            else deto::decompress_dense_kernel<false, false><<<grid, 256, 0, st>>>(
                         p, n, v, val_replica_stride, params, presign_dbg);
        }
        return launched();
    }

    int64_t c0 = 0;
    const int64_t tiles = (n / p.s) / deto::kWave;
    // every replica's array must keep the alignment of a lane's access (four entries when k is
    // a multiple of 4, one element otherwise: the contiguous [R][C*k] layout of an all_gather
    // always qualifies)
    const int64_t ia = static_cast<int64_t>(idx_access(p)), va = static_cast<int64_t>(val_access(p));
    const bool payload_ok =
        aligned(idx, idx_access(p)) && aligned(val, val_access(p)) &&
        (R == 1 ||
         ((!idx || (idx_replica_stride * static_cast<int64_t>(idx_size(idx_dtype))) % ia == 0) &&
          (val_replica_stride * static_cast<int64_t>(val_size(val_dtype))) % va == 0));
    if (tiles <= kMaxTiles && payload_ok && aligned16(params) && aligned16(presign_dbg) &&
        aligned16(adam.m) && aligned16(adam.v) && aligned16(adam.vmax)) {
        deto::DecompressLaunch a{p, tiles, n, C, idx, idx_replica_stride, val,
                                 val_replica_stride, params, param_dtype == DETO_BF16, presign_dbg,
                                 {0, 0, 0, 0}, st, adam};
        stride_pattern(p, a.stride_mask);
        const bool done = tiles == 0 ? false
                          : idx ? (deto::launch_decompress_adamw(a) ||
                                 deto::launch_decompress_adamw_narrow(a) ||
                                 deto::launch_decompress_idx_s64(a) ||
                                 deto::launch_decompress_idx_s32(a) ||
                                 deto::launch_decompress_idx_s16(a) ||
                                 deto::launch_decompress_idx_s96(a) ||
                                 deto::launch_decompress_idx_s128(a) ||
                                 deto::launch_decompress_idx_packed(a) ||
                                 deto::launch_decompress_idx_packed_s32(a) ||
                                 deto::launch_decompress_idx_ternary(a))
                              : (deto::launch_decompress_scheme_adamw(a) ||
                                 deto::launch_decompress_adamw_narrow(a) ||
                                 deto::launch_decompress_scheme(a) ||
                                 deto::launch_decompress_scheme_small(a) ||
                                 deto::launch_decompress_scheme_narrow_s32(a) ||
                                 deto::launch_decompress_scheme_narrow_s64(a));
        if (done) {
            rc = launched();
            if (rc) return rc;
            c0 = C;   // the tail chunks rode along in the same launch
        } else {
            c0 = deto::launch_decompress_split(a);
            if (c0 == 0) c0 = deto::launch_decompress_pair(a);
            if (c0 == 0) c0 = deto::launch_decompress_mfma(a);
            if (c0 > 0) {
                rc = launched();
                if (rc) return rc;
            }
        }
    }
    // Striding in the raw domain without transmitted indices, any chunk size and k
    if (c0 == 0 && !idx && p.scheme == DETO_SCHEME_STRIDE && !p.use_dct && val_dtype == DETO_F32) {
        const deto::StrideGeom sg = deto::stride_geom(p.s, p.k, p.step);
        const int64_t wgs = (n + deto::kStrideSpan - 1) / deto::kStrideSpan;
        if (wgs <= 0x7FFFFFFF) {
            const unsigned grid = static_cast<unsigned>(wgs);
            const float* v = static_cast<const float*>(val);
            if (param_dtype == DETO_BF16)
                deto::decompress_stride_kernel<true><<<grid, 256, 0, st>>>(
                    p, n, sg, v, val_replica_stride, params, adam, presign_dbg);
            else
                deto::decompress_stride_kernel<false><<<grid, 256, 0, st>>>(
                    p, n, sg, v, val_replica_stride, params, adam, presign_dbg);
            return launched();
        }
    }
    if (c0 < C) {
        const unsigned grid = grid_for(C - c0);
        if (param_dtype == DETO_BF16)
            deto::decompress_generic<true><<<grid, deto::kWave, 0, st>>>(
                p, n, c0, C, idx, idx_replica_stride, val, val_replica_stride, params, adam,
                presign_dbg);
        else
            deto::decompress_generic<false><<<grid, deto::kWave, 0, st>>>(
                p, n, c0, C, idx, idx_replica_stride, val, val_replica_stride, params, adam,
                presign_dbg);
        rc = launched();
    }
    return rc;
}

}  // namespace

extern "C" {

int detonation_decompress_step_packed(const deto_config* cfg, int64_t n, int32_t R,
                                      const void* idx, int idx_dtype, int64_t idx_replica_stride,
                                      const void* val, int val_dtype, int64_t val_replica_stride,
                                      void* params, int param_dtype, float* presign_dbg,
                                      void* stream) {
    return decompress_impl(cfg, nullptr, n, R, idx, idx_dtype, idx_replica_stride, val, val_dtype,
                           val_replica_stride, params, param_dtype,
                           deto::AdamPtrs{nullptr, nullptr, nullptr}, presign_dbg, stream);
}

int detonation_decompress_adamw_step(const deto_config* cfg, const deto_adamw* opt, int64_t n,
                                     int32_t R, const int32_t* idx, int64_t idx_replica_stride,
                                     const float* val, int64_t val_replica_stride, void* params,
                                     int param_dtype, float* exp_avg, float* exp_avg_sq,
                                     float* max_exp_avg_sq, float* presign_dbg, void* stream) {
    if (!opt) return DETO_ERR_NULL;
    return decompress_impl(cfg, opt, n, R, idx, DETO_IDX_I32, idx_replica_stride, val, DETO_F32,
                           val_replica_stride, params, param_dtype,
                           deto::AdamPtrs{exp_avg, exp_avg_sq, max_exp_avg_sq}, presign_dbg, stream);
}

int detonation_decompress_adamw_step_packed(const deto_config* cfg, const deto_adamw* opt,
                                            int64_t n, int32_t R, const void* idx, int idx_dtype,
                                            int64_t idx_replica_stride, const void* val,
                                            int val_dtype, int64_t val_replica_stride,
                                            void* params, int param_dtype, float* exp_avg,
                                            float* exp_avg_sq, float* max_exp_avg_sq,
                                            float* presign_dbg, void* stream) {
    if (!opt) return DETO_ERR_NULL;
    return decompress_impl(cfg, opt, n, R, idx, idx_dtype, idx_replica_stride, val, val_dtype,
                           val_replica_stride, params, param_dtype,
                           deto::AdamPtrs{exp_avg, exp_avg_sq, max_exp_avg_sq}, presign_dbg, stream);
}

int detonation_decompress_step(const deto_config* cfg, int64_t n, int32_t R, const int32_t* idx,
                               int64_t idx_replica_stride, const float* val,
                               int64_t val_replica_stride, void* params, int param_dtype,
                               float* presign_dbg, void* stream) {
    return detonation_decompress_step_packed(cfg, n, R, idx, DETO_IDX_I32, idx_replica_stride, val,
                                             DETO_F32, val_replica_stride, params, param_dtype,
                                             presign_dbg, stream);
}

int detonation_accumulate(const deto_config* cfg, int64_t n, const void* grad, int grad_dtype,
                          float* momentum, void* stream) {
    int rc = validate(cfg);
    if (rc) return rc;
    if (n < 0 || !valid_dtype(grad_dtype)) return DETO_ERR_BAD_CONFIG;
    if (n == 0) return DETO_OK;
    if (!grad || !momentum) return DETO_ERR_NULL;
    if (!aligned(grad, elem_size(grad_dtype)) || !aligned(momentum, 4)) return DETO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    fresh_status();
    const bool vec = aligned16(grad) && aligned16(momentum);
    const unsigned grid = stream_grid(n / 8);
    const bool bf16 = grad_dtype == DETO_BF16;
    if (vec && bf16)
        deto::accumulate_kernel<true, true><<<grid, 256, 0, st>>>(cfg->decay, n, grad, momentum);
    else if (vec)
        deto::accumulate_kernel<false, true><<<grid, 256, 0, st>>>(cfg->decay, n, grad, momentum);
    else if (bf16)
        deto::accumulate_kernel<true, false><<<grid, 256, 0, st>>>(cfg->decay, n, grad, momentum);
    else
        deto::accumulate_kernel<false, false><<<grid, 256, 0, st>>>(cfg->decay, n, grad, momentum);
    return launched();
}

int64_t detonation_payload_entries(const deto_config* cfg, int64_t n) {
    if (validate(cfg) != DETO_OK || n < 0) return -1;
    return chunks_of(n, cfg->chunk) * cfg->topk;
}

int64_t detonation_ternary_words(const deto_config* cfg, int64_t n) {
    if (validate(cfg) != DETO_OK || n < 0) return -1;
    return chunks_of(n, cfg->chunk) * ((cfg->topk + 15) / 16);
}

const char* detonation_status_string(int status) {
    switch (status) {
        case DETO_OK: return "ok";
        case DETO_ERR_NULL: return "a required pointer is NULL";
        case DETO_ERR_BAD_CONFIG: return "bad configuration or size";
        case DETO_ERR_UNSUPPORTED: return "unsupported request (more than 64 replicas)";
        case DETO_ERR_ALIGN: return "misaligned pointer";
        case DETO_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

int detonation_version(void) { return 1007; }

}  // extern "C"
