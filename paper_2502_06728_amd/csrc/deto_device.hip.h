// Device-side helpers shared by the gfx950 kernels: dtype conversion, the counter-based
// generator of the Random scheme, kernel parameter block.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace deto {

constexpr int kWave = 64;        // CDNA wavefront width
constexpr int kMaxChunk = 256;   // largest chunk size s the library accepts
constexpr int kMaxReplicas = 64;  // largest replication group R the library accepts

// Everything a kernel needs from deto_config, resolved on the host.
struct KParams {
    int s;              // chunk size
    int k;              // kept entries per chunk
    int scheme;         // deto_scheme
    int use_dct;        // transform domain (always for TOPK)
    int use_sign;       // DETO_FLAG_SIGN
    int R;              // replicas (decompress)
    int val_dtype;      // payload values: 0 fp32, 1 bf16, 2 fp16
    int idx_u8;         // payload indices as bytes instead of int32
    float beta;         // momentum decay
    float lr;           // eta
    float wd_scale;     // 1 - eta*lambda
    float alpha0;       // sqrt(1/s): scale of DCT row 0
    float alpha;        // sqrt(2/s): scale of the other rows
    float inv_R;        // 1/R
    uint64_t seed;
    uint64_t step;
    // Decoupled AdamW as the underlying optimizer (adam != 0)
    int adam;
    int amsgrad;
    float b1, b2;       // betas
    float omb1, omb2;   // 1 - beta
    float eps;
    float step_size;    // eta / (1 - beta1^t)
    float inv_sqrt_bc2; // 1 / sqrt(1 - beta2^t)
};

// AdamW moment arrays (device pointers; vmax only with amsgrad)
struct AdamPtrs {
    float* m;
    float* v;
    float* vmax;
};

// ---- 16-byte global accesses with an optional non-temporal hint.  Every tensor on this
// path is touched once per call; on MI355X the hint lifts a many-stream read from about
// 6.3 to 7.0 TB/s.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// Per-site policy (measured on MI355X, OLMo-1B shard): the decompress kernel gains from
// the hint on every access; the compress kernel, which rewrites the momentum it has just
// read, does not.
#ifndef DETO_NT_COMPRESS_GRAD
#define DETO_NT_COMPRESS_GRAD 0
#endif
#ifndef DETO_NT_COMPRESS_MOM
#define DETO_NT_COMPRESS_MOM 0
#endif
#ifndef DETO_NT_COMPRESS_PAYLOAD
#define DETO_NT_COMPRESS_PAYLOAD 0
#endif
#ifndef DETO_NT_COMPRESS_MOM_ST
#define DETO_NT_COMPRESS_MOM_ST 0
#endif
#ifndef DETO_NT_DECOMPRESS_LD
#define DETO_NT_DECOMPRESS_LD 1
#endif
#ifndef DETO_NT_DECOMPRESS_ST
#define DETO_NT_DECOMPRESS_ST 1
#endif

template <bool NT>
__device__ __forceinline__ float4 ld_f4(const float* p) {
    if constexpr (NT) {
        const f32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
        return make_float4(t.x, t.y, t.z, t.w);
    } else {
        return *reinterpret_cast<const float4*>(p);
    }
}

template <bool NT>
__device__ __forceinline__ uint4 ld_u4(const void* p) {
    if constexpr (NT) {
        const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
        return make_uint4(t.x, t.y, t.z, t.w);
    } else {
        return *reinterpret_cast<const uint4*>(p);
    }
}

typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

template <bool NT>
__device__ __forceinline__ uint2 ld_u2(const void* p) {
    if constexpr (NT) {
        const u32x2_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(p));
        return make_uint2(t.x, t.y);
    } else {
        return *reinterpret_cast<const uint2*>(p);
    }
}

template <bool NT>
__device__ __forceinline__ uint32_t ld_u1(const void* p) {
    if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(p));
    else return *reinterpret_cast<const uint32_t*>(p);
}

template <bool NT>
__device__ __forceinline__ void st_f4(float* p, float4 v) {
    if constexpr (NT) {
        const f32x4_t t = {v.x, v.y, v.z, v.w};
        __builtin_nontemporal_store(t, reinterpret_cast<f32x4_t*>(p));
    } else {
        *reinterpret_cast<float4*>(p) = v;
    }
}

template <bool NT>
__device__ __forceinline__ void st_u4(void* p, uint4 v) {
    if constexpr (NT) {
        const u32x4_t t = {v.x, v.y, v.z, v.w};
        __builtin_nontemporal_store(t, reinterpret_cast<u32x4_t*>(p));
    } else {
        *reinterpret_cast<uint4*>(p) = v;
    }
}

// Ordering point between the LDS phases of a single-wavefront workgroup.  The LDS queue of
// one wavefront is processed in program order, so no hardware barrier is needed; this only
// stops the compiler from moving LDS accesses across the phase boundary.  Unlike
// __syncthreads() it does not wait for outstanding global loads and stores, so prefetched
// data stays in flight and finished tiles retire without waiting for their stores.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// fp32 -> bf16, round to nearest even (finite inputs).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

// IEEE half <-> fp32 (round to nearest even; half subnormals are kept on gfx950)
__device__ __forceinline__ uint16_t f32_to_f16(float f) {
    return __builtin_bit_cast(uint16_t, static_cast<_Float16>(f));
}

__device__ __forceinline__ float f16_to_f32(uint16_t b) {
    return static_cast<float>(__builtin_bit_cast(_Float16, b));
}

// payload value formats: 0 fp32, 1 bf16, 2 fp16
template <int VAL>
__device__ __forceinline__ uint16_t encode16(float v) {
    static_assert(VAL == 1 || VAL == 2, "16-bit transfer dtype");
    if constexpr (VAL == 1) return f32_to_bf16(v);
    else return f32_to_f16(v);
}

template <int VAL>
__device__ __forceinline__ float decode16(uint16_t b) {
    static_assert(VAL == 1 || VAL == 2, "16-bit transfer dtype");
    if constexpr (VAL == 1) return bf16_to_f32(b);
    else return f16_to_f32(b);
}

// two fp32 -> packed bf16 (lo in bits 0..15), round to nearest even: one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// sign(y) in {-1, 0, +1} without compares: scaling by 2^192 (two exact multiplications by
// 2^96, enough to lift the smallest fp32 subnormal above 1) and clamping to [-1, 1] maps
// every non-zero finite y to +-1 and keeps +-0.
__device__ __forceinline__ float sign3(float y) {
    return __builtin_amdgcn_fmed3f(y * 0x1p96f * 0x1p96f, -1.0f, 1.0f);
}

__device__ __forceinline__ float sign_or_self(float y, int use_sign) {
    return use_sign ? sign3(y) : y;
}

// One Decoupled-AdamW step for one element: moments updated in place, returns the new
// parameter value in fp32 (section "Decoupled AdamW"; q is the averaged update).
__device__ __forceinline__ float adamw_step(const KParams& p, float theta, float q, float& m,
                                            float& v, float& vmax) {
    m = fmaf(p.b1, m, p.omb1 * q);
    v = fmaf(p.b2, v, p.omb2 * q * q);
    float vh = v;
    if (p.amsgrad) {
        vmax = fmaxf(vmax, v);
        vh = vmax;
    }
    const float denom = fmaf(sqrtf(vh), p.inv_sqrt_bc2, p.eps);
    return fmaf(-p.step_size, m / denom, theta * p.wd_scale);
}

// ---- Random scheme generator (paper, "Replication Schemes": indices are reproduced on
// every replica from a shared seed).  key = mix64(mix64(seed + G*(step+1)) + G*(chunk+1)),
// draw_j = mix32(lo32(key) + 0x9E3779B9*(j+1)) ^ hi32(key), bounded(d,b) = (d*b) >> 32.
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7FEB352Du;
    x ^= x >> 15;
    x *= 0x846CA68Bu;
    x ^= x >> 16;
    return x;
}

__device__ __forceinline__ uint64_t chunk_key(uint64_t seed, uint64_t step, uint64_t chunk) {
    const uint64_t G = 0x9E3779B97F4A7C15ull;
    return mix64(mix64(seed + G * (step + 1ull)) + G * (chunk + 1ull));
}

__device__ __forceinline__ uint32_t draw(uint64_t key, uint32_t j) {
    return mix32(static_cast<uint32_t>(key) + 0x9E3779B9u * (j + 1u)) ^
           static_cast<uint32_t>(key >> 32);
}

__device__ __forceinline__ uint32_t bounded(uint32_t d, uint32_t b) {
    return __umulhi(d, b);
}

}  // namespace deto
