// Device-side helpers shared by the gfx950 kernels: dtype conversion, the counter-based
// generator of the Random scheme, kernel parameter block.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace deto {

constexpr int kWave = 64;        // CDNA wavefront width
constexpr int kMaxChunk = 256;   // largest chunk size s the library accepts

// Everything a kernel needs from deto_config, resolved on the host.
struct KParams {
    int s;              // chunk size
    int k;              // kept entries per chunk
    int scheme;         // deto_scheme
    int use_dct;        // transform domain (always for TOPK)
    int use_sign;       // DETO_FLAG_SIGN
    int R;              // replicas (decompress)
    float beta;         // momentum decay
    float lr;           // eta
    float wd_scale;     // 1 - eta*lambda
    float alpha0;       // sqrt(1/s): scale of DCT row 0
    float alpha;        // sqrt(2/s): scale of the other rows
    float inv_R;        // 1/R
    uint64_t seed;
    uint64_t step;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// fp32 -> bf16, round to nearest even (finite inputs).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

__device__ __forceinline__ float sign_or_self(float y, int use_sign) {
    if (!use_sign) return y;
    return (y > 0.0f) ? 1.0f : ((y < 0.0f) ? -1.0f : 0.0f);
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
