// General kernels: any chunk size 1..256, any k, every scheme and dtype, ragged last chunk.
// One 64-lane wavefront owns one chunk at a time (lane = element, element e + 64*r for
// longer chunks) and walks the chunk range with a grid stride.  The DCT is the direct
// O(s^2) sum over a cosine table held in LDS.  These kernels cover what the tiled
// kernels do not (odd chunk sizes, the tail of a shard, unaligned buffers); they follow
// Algorithm 1 of the paper step by step.
#pragma once

#include "deto_device.hip.h"

namespace deto {

// cos(pi*t/(2s)) for t in [0, 4s): every DCT-II matrix entry is alpha_j * tab[(2i+1)j mod 4s].
// Only the first quarter period is evaluated (double precision, rounded once); the other three
// follow by symmetry.
__device__ __forceinline__ void build_cos_table(float* tab, int s, int lane) {
    for (int t = lane; t <= s; t += kWave) {
        float c = static_cast<float>(cos(3.14159265358979323846 * static_cast<double>(t) /
                                         (2.0 * static_cast<double>(s))));
        if (t == s) c = 0.0f;
        tab[t] = c;
        tab[2 * s - t] = -c;
        tab[2 * s + t] = -c;
        if (t > 0) tab[4 * s - t] = c;
    }
}

// Striding / Random: flag[e] = 1 for the positions the scheme keeps in chunk `c`.
// Random runs the first k steps of a Fisher-Yates shuffle on one lane.
__device__ __forceinline__ void scheme_flags(const KParams& p, int64_t c, int lane, int* perm,
                                             int* flag) {
    const int s = p.s, k = p.k;
    if (p.scheme == 1) {
        const int stride = s / k;
        const int off = static_cast<int>(p.step % static_cast<uint64_t>(stride));
        for (int e = lane; e < s; e += kWave) {
            const int d = e - off;
            flag[e] = (d >= 0 && d % stride == 0 && d / stride < k) ? 1 : 0;
        }
    } else {
        for (int e = lane; e < s; e += kWave) {
            perm[e] = e;
            flag[e] = 0;
        }
        __syncthreads();
        if (lane == 0) {
            const uint64_t key = chunk_key(p.seed, p.step, static_cast<uint64_t>(c));
            for (int j = 0; j < k; ++j) {
                const int t = j + static_cast<int>(bounded(draw(key, j), s - j));
                const int tmp = perm[j];
                perm[j] = perm[t];
                perm[t] = tmp;
            }
            for (int j = 0; j < k; ++j) flag[perm[j]] = 1;
        }
    }
    __syncthreads();
}

// Turn flags into the ascending list sidx[0..k) (and copy the matching values).
__device__ __forceinline__ void compact_flags(int s, int lane, const int* flag, const float* cf,
                                              int* sidx, float* sval) {
    int before = 0;
    for (int e0 = 0; e0 < s; e0 += kWave) {
        const int e = e0 + lane;
        const bool f = (e < s) && flag[e] != 0;
        const uint64_t mask = __ballot(f);
        const int pos = before + __popcll(mask & ((1ull << lane) - 1ull));
        if (f) {
            sidx[pos] = e;
            if (cf) sval[pos] = cf[e];
        }
        before += __popcll(mask);
    }
    __syncthreads();
}

// Payload access in whatever format the caller chose (runtime switch: these kernels are the
// general path).  What the momentum gives up for a kept coefficient v: the value the receivers
// decode for the 16-bit formats; v itself for fp32 and for the ternary payload (Algorithm 1:
// the extracted components leave the momentum, whatever goes on the wire).
__device__ __forceinline__ float payload_roundtrip(int val_dtype, float v) {
    if (val_dtype == 1) return decode16<1>(encode16<1>(v));
    if (val_dtype == 2) return decode16<2>(encode16<2>(v));
    return v;
}

// ---- ternary payload: sign(v) in two bits (0 = zero, 1 = +1, 3 = -1), 16 entries per 32-bit
// word, every chunk on a word boundary (ceil(k/16) words per chunk).
__device__ __forceinline__ int ternary_words_per_chunk(int k) { return (k + 15) >> 4; }

// bit i of x (i < 16) -> bit 2i
__device__ __forceinline__ uint32_t spread16(uint32_t x) {
    x = (x | (x << 8)) & 0x00FF00FFu;
    x = (x | (x << 4)) & 0x0F0F0F0Fu;
    x = (x | (x << 2)) & 0x33333333u;
    x = (x | (x << 1)) & 0x55555555u;
    return x;
}

__device__ __forceinline__ float ternary_decode(uint32_t word, int j) {
    const uint32_t code = (word >> (2 * (j & 15))) & 3u;
    return (code & 1u) ? ((code & 2u) ? -1.0f : 1.0f) : 0.0f;
}

// The k kept values of one chunk, sval[0..k) in LDS, to the chunk's words (whole wavefront).
__device__ __forceinline__ void store_ternary_chunk(uint32_t* __restrict__ words, int k, int lane,
                                                    const float* sval) {
    for (int j0 = 0; j0 < k; j0 += kWave) {
        const int j = j0 + lane;
        const float v = (j < k) ? sval[j] : 0.0f;
        const uint64_t nz = __ballot(v != 0.0f);
        const uint64_t ng = __ballot(v < 0.0f);
        if (lane < 4 && j0 + 16 * lane < k) {
            const uint32_t a = static_cast<uint32_t>(nz >> (16 * lane)) & 0xFFFFu;
            const uint32_t b = static_cast<uint32_t>(ng >> (16 * lane)) & 0xFFFFu;
            words[(j0 >> 4) + lane] = spread16(a) | (spread16(b) << 1);
        }
    }
}

__device__ __forceinline__ void store_payload_value(void* base, int64_t e, int val_dtype, float v) {
    if (val_dtype == 0) static_cast<float*>(base)[e] = v;
    else static_cast<uint16_t*>(base)[e] = (val_dtype == 1) ? encode16<1>(v) : encode16<2>(v);
}

__device__ __forceinline__ float load_payload_value(const void* base, int64_t e, int val_dtype) {
    if (val_dtype == 0) return static_cast<const float*>(base)[e];
    const uint16_t b = static_cast<const uint16_t*>(base)[e];
    return (val_dtype == 1) ? decode16<1>(b) : decode16<2>(b);
}

__device__ __forceinline__ void store_payload_index(void* base, int64_t e, int idx_u8, int at) {
    if (idx_u8) static_cast<uint8_t*>(base)[e] = static_cast<uint8_t>(at);
    else static_cast<int32_t*>(base)[e] = at;
}

__device__ __forceinline__ int load_payload_index(const void* base, int64_t e, int idx_u8) {
    return idx_u8 ? static_cast<int>(static_cast<const uint8_t*>(base)[e])
                  : static_cast<const int32_t*>(base)[e];
}

// LDS working set of one wavefront of the general compress / decompress code.
struct GenericCompressSmem {
    float tab[4 * kMaxChunk];
    float x[kMaxChunk];
    float cf[kMaxChunk];
    float sval[kMaxChunk];
    int flag[kMaxChunk];
    int sidx[kMaxChunk];
    int perm[kMaxChunk];
};

struct GenericDecompressSmem {
    float tab[4 * kMaxChunk];
    float a[kMaxChunk];
    int flag[kMaxChunk];
    int sidx[kMaxChunk];
    int perm[kMaxChunk];
};

// Compress half for the chunks first, first+stride, ... below chunk_end, one chunk at a time
// on the calling wavefront.  Also the tail path of the tiled kernels (the chunks that do not
// fill a tile), which call it from their surplus workgroups.
template <bool GRAD_BF16>
__device__ __forceinline__ void compress_generic_chunks(
    const KParams& p, int64_t n, int64_t first, int64_t chunk_end, int64_t stride,
    GenericCompressSmem& sm, const void* __restrict__ grad, float* __restrict__ mom,
    void* __restrict__ idx_out, void* __restrict__ val_out, float* __restrict__ coeff_dbg) {
    float* tab = sm.tab;
    float* x = sm.x;
    float* cf = sm.cf;
    float* sval = sm.sval;
    int* flag = sm.flag;
    int* sidx = sm.sidx;
    int* perm = sm.perm;

    const int lane = threadIdx.x;
    const int s = p.s, k = p.k;
    if (p.use_dct) build_cos_table(tab, s, lane);
    __syncthreads();

    for (int64_t c = first; c < chunk_end; c += stride) {
        const int64_t base = c * s;
        // m1 = beta*m + g, zero beyond the shard
        for (int e = lane; e < s; e += kWave) {
            const int64_t i = base + e;
            float v = 0.0f;
            if (i < n) {
                const float g = GRAD_BF16 ? bf16_to_f32(static_cast<const uint16_t*>(grad)[i])
                                          : static_cast<const float*>(grad)[i];
                v = fmaf(p.beta, mom[i], g);
            }
            x[e] = v;
        }
        __syncthreads();
        // coefficients
        for (int e = lane; e < s; e += kWave) {
            float acc;
            if (p.use_dct) {
                acc = 0.0f;
                int ph = e;
                // (unrolled so that the LDS reads of several terms are in flight together; the
                // additions keep their order)
#pragma unroll 8
                for (int t = 0; t < s; ++t) {
                    acc = fmaf(x[t], tab[ph], acc);
                    ph += 2 * e;
                    if (ph >= 4 * s) ph -= 4 * s;
                }
                acc *= (e == 0) ? p.alpha0 : p.alpha;
            } else {
                acc = x[e];
            }
            cf[e] = acc;
            if (coeff_dbg) coeff_dbg[base + e] = acc;
        }
        __syncthreads();
        // which entries are kept
        if (p.scheme == 0) {
            for (int e = lane; e < s; e += kWave) {
                const uint32_t me = __float_as_uint(cf[e]) & 0x7FFFFFFFu;
                int rank = 0;
#pragma unroll 8
                for (int t = 0; t < s; ++t) {
                    const uint32_t o = __float_as_uint(cf[t]) & 0x7FFFFFFFu;
                    rank += (o > me || (o == me && t < e)) ? 1 : 0;
                }
                flag[e] = rank < k ? 1 : 0;
            }
            __syncthreads();
        } else {
            scheme_flags(p, c, lane, perm, flag);
        }
        compact_flags(s, lane, flag, cf, sidx, sval);
        // what travels is the value in the transfer dtype; the residual below removes exactly
        // what the receivers will decode
        if (p.val_dtype == 3)
            store_ternary_chunk(static_cast<uint32_t*>(val_out) + c * ternary_words_per_chunk(k), k,
                                lane, sval);
        for (int j = lane; j < k; j += kWave) {
            if (idx_out) store_payload_index(idx_out, c * k + j, p.idx_u8, sidx[j]);
            if (p.val_dtype != 3) store_payload_value(val_out, c * k + j, p.val_dtype, sval[j]);
            sval[j] = payload_roundtrip(p.val_dtype, sval[j]);
        }
        __syncthreads();
        // m <- m1 - q
        for (int e = lane; e < s; e += kWave) {
            const int64_t i = base + e;
            if (i >= n) continue;
            float q;
            if (p.use_dct) {
                q = 0.0f;
#pragma unroll 4
                for (int j = 0; j < k; ++j) {
                    const int r = sidx[j];
                    const float a = (r == 0) ? p.alpha0 : p.alpha;
                    q = fmaf(tab[((2 * e + 1) * r) % (4 * s)], a * sval[j], q);
                }
            } else {
                q = flag[e] ? payload_roundtrip(p.val_dtype, x[e]) : 0.0f;
            }
            mom[i] = x[e] - q;
        }
        __syncthreads();
    }
}

template <bool GRAD_BF16>
__global__ __launch_bounds__(kWave) void compress_generic(KParams p, int64_t n,
                                                          int64_t chunk_begin, int64_t chunk_end,
                                                          const void* __restrict__ grad,
                                                          float* __restrict__ mom,
                                                          void* __restrict__ idx_out,
                                                          void* __restrict__ val_out,
                                                          float* __restrict__ coeff_dbg) {
    __shared__ GenericCompressSmem sm;
    compress_generic_chunks<GRAD_BF16>(p, n, chunk_begin + blockIdx.x, chunk_end, gridDim.x, sm,
                                       grad, mom, idx_out, val_out, coeff_dbg);
}

// Decompress-and-update half for the chunks first, first+stride, ... below chunk_end.
template <bool PARAM_BF16>
__device__ __forceinline__ void decompress_generic_chunks(
    const KParams& p, int64_t n, int64_t first, int64_t chunk_end, int64_t stride,
    GenericDecompressSmem& sm, const void* __restrict__ idx, int64_t idx_stride,
    const void* __restrict__ val, int64_t val_stride, void* __restrict__ params,
    const AdamPtrs& ad, float* __restrict__ presign_dbg) {
    float* tab = sm.tab;
    float* a = sm.a;
    int* flag = sm.flag;
    int* sidx = sm.sidx;
    int* perm = sm.perm;

    const int lane = threadIdx.x;
    const int s = p.s, k = p.k;
    if (p.use_dct) build_cos_table(tab, s, lane);
    __syncthreads();

    for (int64_t c = first; c < chunk_end; c += stride) {
        const int64_t base = c * s;
        for (int e = lane; e < s; e += kWave) a[e] = 0.0f;
        if (!idx) {
            scheme_flags(p, c, lane, perm, flag);
            compact_flags(s, lane, flag, nullptr, sidx, nullptr);
        } else {
            __syncthreads();
        }
        // scatter-add, one replica after the other so the order of additions is fixed.  An
        // entry's index and value are requested together, and (k <= 64: one entry per lane)
        // those of four replicas before the first is added.
        auto entry = [&](int r, int j, int& at, float& v) {
            at = idx ? load_payload_index(idx, r * idx_stride + c * k + j, p.idx_u8) : sidx[j];
            v = (p.val_dtype == 3)
                    ? ternary_decode(static_cast<const uint32_t*>(
                                         val)[r * val_stride + c * ternary_words_per_chunk(k) +
                                              (j >> 4)], j)
                    : load_payload_value(val, r * val_stride + c * k + j, p.val_dtype);
        };
        if (k <= kWave) {
            constexpr int kBatch = 4;
            for (int r0 = 0; r0 < p.R; r0 += kBatch) {
                int at[kBatch];
                float v[kBatch];
#pragma unroll
                for (int b = 0; b < kBatch; ++b) {
                    at[b] = -1;
                    v[b] = 0.0f;
                    if (r0 + b < p.R && lane < k) entry(r0 + b, lane, at[b], v[b]);
                }
#pragma unroll
                for (int b = 0; b < kBatch; ++b) {
                    if (r0 + b < p.R) {
                        if (at[b] >= 0 && at[b] < s) atomicAdd(&a[at[b]], v[b]);
                        __syncthreads();
                    }
                }
            }
        } else {
            for (int r = 0; r < p.R; ++r) {
                for (int j = lane; j < k; j += kWave) {
                    int at;
                    float v;
                    entry(r, j, at, v);
                    if (at >= 0 && at < s) atomicAdd(&a[at], v);
                }
                __syncthreads();
            }
        }
        if (p.use_dct) {
            // the averaged coefficients with their scale factors, once per chunk
            for (int e = lane; e < s; e += kWave)
                a[e] = ((e == 0) ? p.alpha0 : p.alpha) * (a[e] * p.inv_R);
            __syncthreads();
        }
        for (int e = lane; e < s; e += kWave) {
            const int64_t i = base + e;
            if (i >= n) continue;
            float y;
            if (p.use_dct) {
                // y_e = sum_j tab[(2e+1) j mod 4s] a_j, the table position kept in bytes
                y = 0.0f;
                const uint32_t period = 16u * static_cast<uint32_t>(s);
                const uint32_t step = 4u * static_cast<uint32_t>(2 * e + 1);
                const char* tab_bytes = reinterpret_cast<const char*>(tab);
                uint32_t ph = 0u;
#pragma unroll 8
                for (int j = 0; j < s; ++j) {
                    y = fmaf(*reinterpret_cast<const float*>(tab_bytes + ph), a[j], y);
                    ph += step;
                    ph = min(ph, ph - period);      // ph -= period where ph >= period
                }
            } else {
                y = a[e] * p.inv_R;
            }
            if (presign_dbg) presign_dbg[i] = y;
            const float q = sign_or_self(y, p.use_sign);
            const float old = PARAM_BF16 ? bf16_to_f32(static_cast<uint16_t*>(params)[i])
                                         : static_cast<float*>(params)[i];
            float nw;
            if (p.adam) {
                float m = ad.m[i], v = ad.v[i], vm = p.amsgrad ? ad.vmax[i] : 0.0f;
                nw = adamw_step(p, old, q, m, v, vm);
                ad.m[i] = m;
                ad.v[i] = v;
                if (p.amsgrad) ad.vmax[i] = vm;
            } else {
                nw = fmaf(-p.lr, q, old * p.wd_scale);
            }
            if (PARAM_BF16) static_cast<uint16_t*>(params)[i] = f32_to_bf16(nw);
            else static_cast<float*>(params)[i] = nw;
        }
        __syncthreads();
    }
}

template <bool PARAM_BF16>
__global__ __launch_bounds__(kWave) void decompress_generic(
    KParams p, int64_t n, int64_t chunk_begin, int64_t chunk_end, const void* __restrict__ idx,
    int64_t idx_stride, const void* __restrict__ val, int64_t val_stride,
    void* __restrict__ params, AdamPtrs ad, float* __restrict__ presign_dbg) {
    __shared__ GenericDecompressSmem sm;
    decompress_generic_chunks<PARAM_BF16>(p, n, chunk_begin + blockIdx.x, chunk_end, gridDim.x, sm,
                                          idx, idx_stride, val, val_stride, params, ad,
                                          presign_dbg);
}

// m <- beta*m + g over the whole shard (Algorithm 1, first line), nothing else: eight
// elements per lane and iteration with 16-byte accesses when the buffers allow it.
template <bool GRAD_BF16, bool VEC>
__global__ __launch_bounds__(256) void accumulate_kernel(float beta, int64_t n,
                                                         const void* __restrict__ grad,
                                                         float* __restrict__ mom) {
    const int64_t tid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t nthreads = static_cast<int64_t>(gridDim.x) * blockDim.x;
    int64_t done = 0;
    if constexpr (VEC) {
        const int64_t groups = n / 8;
        for (int64_t q = tid; q < groups; q += nthreads) {
            const int64_t e = 8 * q;
            float g[8];
            if constexpr (GRAD_BF16) {
                const uint4 raw = ld_u4<true>(static_cast<const uint16_t*>(grad) + e);
                const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    g[2 * j] = __uint_as_float(w[j] << 16);
                    g[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
                }
            } else {
                const float4 a = ld_f4<true>(static_cast<const float*>(grad) + e);
                const float4 b = ld_f4<true>(static_cast<const float*>(grad) + e + 4);
                g[0] = a.x; g[1] = a.y; g[2] = a.z; g[3] = a.w;
                g[4] = b.x; g[5] = b.y; g[6] = b.z; g[7] = b.w;
            }
            const float4 ma = ld_f4<false>(mom + e), mb = ld_f4<false>(mom + e + 4);
            st_f4<false>(mom + e, make_float4(fmaf(beta, ma.x, g[0]), fmaf(beta, ma.y, g[1]),
                                              fmaf(beta, ma.z, g[2]), fmaf(beta, ma.w, g[3])));
            st_f4<false>(mom + e + 4, make_float4(fmaf(beta, mb.x, g[4]), fmaf(beta, mb.y, g[5]),
                                                  fmaf(beta, mb.z, g[6]), fmaf(beta, mb.w, g[7])));
        }
        done = groups * 8;
    }
    for (int64_t i = done + tid; i < n; i += nthreads) {
        const float g = GRAD_BF16 ? bf16_to_f32(static_cast<const uint16_t*>(grad)[i])
                                  : static_cast<const float*>(grad)[i];
        mom[i] = fmaf(beta, mom[i], g);
    }
}

// ---- k = s in the raw domain (Striding or Random that keep every position: the synchronising
// step of a DiLoCo cycle): the payload is the whole folded momentum and the momentum restarts
// from zero; the receivers average R dense arrays.  Plain streaming kernels, four elements per
// lane and iteration with 16-byte accesses when the buffers allow it.
template <bool GRAD_BF16, bool VEC>
__global__ __launch_bounds__(256) void compress_dense_kernel(KParams p, int64_t n, int64_t entries,
                                                             const void* __restrict__ grad,
                                                             float* __restrict__ mom,
                                                             int32_t* __restrict__ idx_out,
                                                             float* __restrict__ val_out,
                                                             float* __restrict__ coeff_dbg) {
    const int64_t tid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t nthreads = static_cast<int64_t>(gridDim.x) * blockDim.x;
    int64_t done = 0;
    if constexpr (VEC) {
        const int64_t groups = n / 4;
        for (int64_t q = tid; q < groups; q += nthreads) {
            const int64_t e = 4 * q;
            float4 g;
            if constexpr (GRAD_BF16) {
                const uint2 raw = ld_u2<true>(static_cast<const uint16_t*>(grad) + e);
                g = make_float4(__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xFFFF0000u),
                                __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xFFFF0000u));
            } else {
                g = ld_f4<true>(static_cast<const float*>(grad) + e);
            }
            const float4 m = ld_f4<false>(mom + e);
            const float4 v = make_float4(fmaf(p.beta, m.x, g.x), fmaf(p.beta, m.y, g.y),
                                         fmaf(p.beta, m.z, g.z), fmaf(p.beta, m.w, g.w));
            st_f4<false>(val_out + e, v);
            st_f4<false>(mom + e, make_float4(0.0f, 0.0f, 0.0f, 0.0f));
            if (coeff_dbg) st_f4<false>(coeff_dbg + e, v);
            if (idx_out) {
                const int at = static_cast<int>(e % p.s);      // s is a multiple of 4 here
                *reinterpret_cast<int4*>(idx_out + e) = make_int4(at, at + 1, at + 2, at + 3);
            }
        }
        done = groups * 4;
    }
    // the elements the vector loop did not take, and the zero-extension of the last chunk
    for (int64_t e = done + tid; e < entries; e += nthreads) {
        float v = 0.0f;
        if (e < n) {
            const float g = GRAD_BF16 ? bf16_to_f32(static_cast<const uint16_t*>(grad)[e])
                                      : static_cast<const float*>(grad)[e];
            v = fmaf(p.beta, mom[e], g);
            mom[e] = 0.0f;
        }
        val_out[e] = v;
        if (coeff_dbg) coeff_dbg[e] = v;
        if (idx_out) idx_out[e] = static_cast<int32_t>(e % p.s);
    }
}

template <bool PARAM_BF16, bool VEC>
__global__ __launch_bounds__(256) void decompress_dense_kernel(KParams p, int64_t n,
                                                               const float* __restrict__ val,
                                                               int64_t val_stride,
                                                               void* __restrict__ params,
                                                               float* __restrict__ presign_dbg) {
    const int64_t tid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t nthreads = static_cast<int64_t>(gridDim.x) * blockDim.x;
    int64_t done = 0;
    if constexpr (VEC) {
        const int64_t groups = n / 4;
        for (int64_t q = tid; q < groups; q += nthreads) {
            const int64_t e = 4 * q;
            float4 a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            for (int r = 0; r < p.R; ++r) {           // replica after replica: a fixed order
                const float4 v = ld_f4<true>(val + r * val_stride + e);
                a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
            }
            const float y[4] = {a.x * p.inv_R, a.y * p.inv_R, a.z * p.inv_R, a.w * p.inv_R};
            if (presign_dbg) st_f4<false>(presign_dbg + e, make_float4(y[0], y[1], y[2], y[3]));
            float nw[4], old[4];
            if constexpr (PARAM_BF16) {
                const uint2 raw = ld_u2<true>(static_cast<const uint16_t*>(params) + e);
                old[0] = __uint_as_float(raw.x << 16);
                old[1] = __uint_as_float(raw.x & 0xFFFF0000u);
                old[2] = __uint_as_float(raw.y << 16);
                old[3] = __uint_as_float(raw.y & 0xFFFF0000u);
            } else {
                const float4 o = ld_f4<true>(static_cast<const float*>(params) + e);
                old[0] = o.x; old[1] = o.y; old[2] = o.z; old[3] = o.w;
            }
#pragma unroll
            for (int c = 0; c < 4; ++c)
                nw[c] = fmaf(-p.lr, sign_or_self(y[c], p.use_sign), old[c] * p.wd_scale);
            if constexpr (PARAM_BF16) {
                *reinterpret_cast<uint2*>(static_cast<uint16_t*>(params) + e) =
                    make_uint2(pack_bf16x2(nw[0], nw[1]), pack_bf16x2(nw[2], nw[3]));
            } else {
                st_f4<false>(static_cast<float*>(params) + e,
                             make_float4(nw[0], nw[1], nw[2], nw[3]));
            }
        }
        done = groups * 4;
    }
    for (int64_t i = done + tid; i < n; i += nthreads) {
        float a = 0.0f;
        for (int r = 0; r < p.R; ++r) a += val[r * val_stride + i];
        const float y = a * p.inv_R;
        if (presign_dbg) presign_dbg[i] = y;
        const float old = PARAM_BF16 ? bf16_to_f32(static_cast<uint16_t*>(params)[i])
                                     : static_cast<float*>(params)[i];
        const float nw = fmaf(-p.lr, sign_or_self(y, p.use_sign), old * p.wd_scale);
        if (PARAM_BF16) static_cast<uint16_t*>(params)[i] = f32_to_bf16(nw);
        else static_cast<float*>(params)[i] = nw;
    }
}

// ---- Striding in the raw domain at any chunk size and k (paper, "Replication Schemes": the
// selection of every n-th position; it does not look at the values, so nothing per chunk needs
// computing): plain streaming kernels, one workgroup of 256 lanes per kStrideSpan consecutive
// elements, every access a coalesced lane access of one element (no alignment beyond the
// element size is needed).  Position r of chunk c is kept when r = o + j*stride for some
// j < k and then becomes entry j of the chunk.  The shapes the lane-per-chunk kernels serve
// run there.
constexpr int kStrideSpan = 2048;

struct StridePos {
    int64_t chunk;
    int r;        // position in the chunk
    int j;        // entry number if kept
    bool kept;
};

// Divisions by the chunk size and by the stride as multiply-and-shift, exact for the small
// numerators that occur: t < s + kStrideSpan <= 2304 with ceil(2^20/s) (the error term
// t*(m*s - 2^20) stays below 2^20 for s <= 256), d < 256 with ceil(2^16/stride).
struct StrideGeom {
    int stride;
    int off;
    uint32_t chunk_magic;    // ceil(2^20 / s)
    uint32_t stride_magic;   // ceil(2^16 / stride)
};

__host__ __device__ inline StrideGeom stride_geom(int s, int k, uint64_t step) {
    StrideGeom g;
    g.stride = s / k;
    g.off = static_cast<int>(step % static_cast<uint64_t>(g.stride));
    g.chunk_magic = ((1u << 20) + static_cast<uint32_t>(s) - 1u) / static_cast<uint32_t>(s);
    g.stride_magic =
        ((1u << 16) + static_cast<uint32_t>(g.stride) - 1u) / static_cast<uint32_t>(g.stride);
    return g;
}

__device__ __forceinline__ StridePos stride_position(const KParams& p, const StrideGeom& sg,
                                                     int64_t c_base, int r_base, int local) {
    const uint32_t t = static_cast<uint32_t>(r_base + local);
    const uint32_t dc = (t * sg.chunk_magic) >> 20;
    StridePos q;
    q.chunk = c_base + dc;
    q.r = static_cast<int>(t - dc * static_cast<uint32_t>(p.s));
    const int d = q.r - sg.off;
    q.j = d >= 0 ? static_cast<int>((static_cast<uint32_t>(d) * sg.stride_magic) >> 16) : 0;
    q.kept = d >= 0 && q.j * sg.stride == d && q.j < p.k;
    return q;
}

template <bool GRAD_BF16>
__global__ __launch_bounds__(256) void compress_stride_kernel(
    KParams p, int64_t n, int64_t padded, StrideGeom sg, const void* __restrict__ grad,
    float* __restrict__ mom, int32_t* __restrict__ idx_out, float* __restrict__ val_out,
    float* __restrict__ coeff_dbg) {
    constexpr int kIt = kStrideSpan / 256;
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kStrideSpan;
    const int64_t c_base = base / p.s;
    const int r_base = static_cast<int>(base - c_base * p.s);
    // all loads of the workgroup's span first
    float g[kIt], m[kIt];
#pragma unroll
    for (int q = 0; q < kIt; ++q) {
        const int64_t i = base + threadIdx.x + 256 * q;
        g[q] = 0.0f;
        m[q] = 0.0f;
        if (i < n) {
            g[q] = GRAD_BF16 ? bf16_to_f32(static_cast<const uint16_t*>(grad)[i])
                             : static_cast<const float*>(grad)[i];
            m[q] = mom[i];
        }
    }
#pragma unroll
    for (int q = 0; q < kIt; ++q) {
        const int local = threadIdx.x + 256 * q;
        const int64_t i = base + local;
        if (i < padded) {       // positions n <= i < padded: the zero-extension of the last chunk
            const float v = i < n ? fmaf(p.beta, m[q], g[q]) : 0.0f;
            const StridePos at = stride_position(p, sg, c_base, r_base, local);
            if (at.kept) {
                const int64_t e = at.chunk * p.k + at.j;
                val_out[e] = v;
                if (idx_out) idx_out[e] = at.r;
            }
            if (i < n) mom[i] = at.kept ? 0.0f : v;
            if (coeff_dbg) coeff_dbg[i] = v;
        }
    }
}

template <bool PARAM_BF16>
__global__ __launch_bounds__(256) void decompress_stride_kernel(
    KParams p, int64_t n, StrideGeom sg, const float* __restrict__ val, int64_t val_stride,
    void* __restrict__ params, AdamPtrs ad, float* __restrict__ presign_dbg) {
    constexpr int kIt = kStrideSpan / 256;
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kStrideSpan;
    const int64_t c_base = base / p.s;
    const int r_base = static_cast<int>(base - c_base * p.s);
    // the parameters and, replica after replica, the kept positions' values of the whole span
    // are requested side by side (the eight elements of a lane are independent)
    float old[kIt], a[kIt];
    int64_t entry[kIt];          // the position's payload entry, -1 if it is not kept
#pragma unroll
    for (int q = 0; q < kIt; ++q) {
        const int local = threadIdx.x + 256 * q;
        const int64_t i = base + local;
        old[q] = 0.0f;
        a[q] = 0.0f;
        entry[q] = -1;
        if (i < n) {
            old[q] = PARAM_BF16 ? bf16_to_f32(static_cast<const uint16_t*>(params)[i])
                                : static_cast<const float*>(params)[i];
            const StridePos at = stride_position(p, sg, c_base, r_base, local);
            if (at.kept) entry[q] = at.chunk * p.k + at.j;
        }
    }
    // unconditional loads (entry 0 stands in for positions that are not kept) so that the
    // eight of a replica are requested together; a load under a branch is waited for there
    for (int r = 0; r < p.R; ++r) {           // replica after replica: a fixed order
        const float* v = val + r * val_stride;
        float x[kIt];
#pragma unroll
        for (int q = 0; q < kIt; ++q) x[q] = v[entry[q] >= 0 ? entry[q] : 0];
#pragma unroll
        for (int q = 0; q < kIt; ++q) a[q] += entry[q] >= 0 ? x[q] : 0.0f;
    }
#pragma unroll
    for (int q = 0; q < kIt; ++q) {
        const int64_t i = base + threadIdx.x + 256 * q;
        if (i < n) {
            const float y = entry[q] >= 0 ? a[q] * p.inv_R : 0.0f;
            if (presign_dbg) presign_dbg[i] = y;
            const float qv = sign_or_self(y, p.use_sign);
            float nw;
            if (p.adam) {
                float m1 = ad.m[i], v1 = ad.v[i], x1 = p.amsgrad ? ad.vmax[i] : 0.0f;
                nw = adamw_step(p, old[q], qv, m1, v1, x1);
                ad.m[i] = m1;
                ad.v[i] = v1;
                if (p.amsgrad) ad.vmax[i] = x1;
            } else {
                nw = fmaf(-p.lr, qv, old[q] * p.wd_scale);
            }
            if constexpr (PARAM_BF16) static_cast<uint16_t*>(params)[i] = f32_to_bf16(nw);
            else static_cast<float*>(params)[i] = nw;
        }
    }
}

}  // namespace deto
