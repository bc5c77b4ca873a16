// Host-side launchers of the tiled kernels.  Each translation unit tiled_*.hip instantiates
// one family of kernels and defines its launcher, so the families compile in parallel.
// A launcher returns true if it has a kernel for (p.s, p.k) and has enqueued it.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "deto_device.hip.h"

namespace deto {

struct CompressLaunch {
    KParams p;
    int64_t tiles;          // full 64-chunk tiles, one workgroup each
    int64_t n;              // shard length
    int64_t n_chunks;       // ceil(n / s): the chunks past the last full tile ride along
    const void* grad;
    bool grad_bf16;
    float* mom;
    void* idx;              // may be null for Striding/Random; dtype per p.idx_u8
    void* val;              // dtype per p.val_dtype
    float* coeff_dbg;
    uint32_t stride_mask[4];  // Striding: kept positions of every chunk (bit i%32 of word i/32)
    hipStream_t stream;
};

struct DecompressLaunch {
    KParams p;
    int64_t tiles;
    int64_t n;
    int64_t n_chunks;
    const void* idx;        // null: indices regenerated from the scheme
    int64_t idx_stride;     // replica strides in elements
    const void* val;
    int64_t val_stride;
    void* params;
    bool param_bf16;
    float* presign_dbg;
    uint32_t stride_mask[4];
    hipStream_t stream;
    AdamPtrs adam;          // moment arrays when p.adam
};

// A shard of at most this many 64-chunk tiles counts as small: the launch is a few occupancy
// rounds long, so what a tile takes from its first load to its last store decides the duration,
// not the instructions per element.  The compress half then spreads a tile over more wavefronts
// (chunk 64: two coefficient classes instead of a lane per chunk; chunk 128: four instead of
// two).  Measured on MI355X: 4 - 13 % shorter launches at 1,300 - 8,000 tiles, 4 - 5 % longer
// ones at 36,000.  The environment variable DETO_SMALL_SHARD_TILES overrides the limit (0: never).
inline int64_t small_shard_tiles() {
    const char* e = getenv("DETO_SMALL_SHARD_TILES");
    if (e && *e) {
        char* end = nullptr;
        const long long v = strtoll(e, &end, 10);
        if (end != e && v >= 0) return static_cast<int64_t>(v);
    }
    return 8192;
}

// grid of a launch: one workgroup per tile plus one per tail chunk
inline unsigned tiled_grid(int64_t tiles, int64_t n_chunks) {
    return static_cast<unsigned>(tiles + (n_chunks - tiles * kWave));
}

bool launch_compress_topk_s64(const CompressLaunch& a);
bool launch_compress_topk_s32(const CompressLaunch& a);
bool launch_compress_topk_s16(const CompressLaunch& a);
bool launch_decompress_idx_s64(const DecompressLaunch& a);
bool launch_decompress_idx_s32(const DecompressLaunch& a);
bool launch_decompress_idx_s16(const DecompressLaunch& a);
bool launch_decompress_idx_s96(const DecompressLaunch& a);
bool launch_decompress_idx_s128(const DecompressLaunch& a);
bool launch_compress_topk_packed(const CompressLaunch& a);     // byte indices + 16-bit values
bool launch_decompress_idx_packed(const DecompressLaunch& a);
bool launch_compress_topk_packed_s32(const CompressLaunch& a);
bool launch_decompress_idx_packed_s32(const DecompressLaunch& a);
bool launch_compress_topk_ternary(const CompressLaunch& a);    // byte indices + two-bit signs
bool launch_decompress_idx_ternary(const DecompressLaunch& a);
bool launch_decompress_adamw(const DecompressLaunch& a);       // Decoupled AdamW update
bool launch_decompress_adamw_narrow(const DecompressLaunch& a);   // ... narrow payloads, with or without indices
bool launch_decompress_scheme_adamw(const DecompressLaunch& a);   // ... without transmitted indices
bool launch_compress_scheme_narrow_s32(const CompressLaunch& a);   // Striding / Random, narrow payload
bool launch_decompress_scheme_narrow_s32(const DecompressLaunch& a);
bool launch_compress_scheme_narrow_s64(const CompressLaunch& a);
bool launch_decompress_scheme_narrow_s64(const DecompressLaunch& a);
bool launch_compress_scheme(const CompressLaunch& a);
bool launch_decompress_scheme(const DecompressLaunch& a);
bool launch_compress_scheme_small(const CompressLaunch& a);    // low compression rates
bool launch_decompress_scheme_small(const DecompressLaunch& a);

// Matrix-core kernels: tiles of 32 complete chunks, persistent single-wavefront workgroups.
// A launcher returns the number of leading chunks it has taken (0: no kernel for this request).
#ifdef DETO_TILED_ONLY_64_32
#define DETO_MFMA_NB_LIST(X) X(4)
#else
#define DETO_MFMA_NB_LIST(X) X(1) X(2) X(3) X(4) X(5) X(7)   // 6 and 8: two-lanes-per-chunk kernels
#endif

inline unsigned mfma_grid(int64_t tiles, size_t smem_bytes) {
    const int64_t per_cu = static_cast<int64_t>((160u * 1024u) / smem_bytes);   // LDS-limited
    const int64_t cap = 256 * (per_cu < 8 ? per_cu : 8);
    return static_cast<unsigned>(tiles < cap ? tiles : cap);
}

int64_t launch_compress_mfma(const CompressLaunch& a);
int64_t launch_decompress_mfma(const DecompressLaunch& a);

// Two-lanes-per-chunk kernels (register-resident fast DCT split between lanes t and t+32): the
// chunk sizes that do not fit one lane.  Same tiles and return convention.
#ifdef DETO_TILED_ONLY_64_32
#define DETO_PAIR_S_LIST(X)
#else
#define DETO_PAIR_S_LIST(X) X(192) X(256)
#endif
int64_t launch_compress_pair_96(const CompressLaunch& a);    // one translation unit each:
int64_t launch_compress_pair_128(const CompressLaunch& a);   // the longest compiles
int64_t launch_compress_pair_192(const CompressLaunch& a);
int64_t launch_compress_pair_256(const CompressLaunch& a);
inline int64_t launch_compress_pair(const CompressLaunch& a) {
    int64_t c = launch_compress_pair_96(a);
    if (!c) c = launch_compress_pair_128(a);
    if (!c) c = launch_compress_pair_192(a);
    return c ? c : launch_compress_pair_256(a);
}
int64_t launch_decompress_pair(const DecompressLaunch& a);

// Lane per chunk, wavefront per coefficient class (split_kernels.hip.h): tiles of 64 chunks,
// fp32 + int32 payloads with k <= s/2.  Same return convention.
int64_t launch_decompress_split(const DecompressLaunch& a);      // chunk 192, 256; 64, 96, 128 at other k
// chunk 64 on a small shard only (see small_shard_tiles); tried before the lane-per-chunk kernel
int64_t launch_compress_split_64(const CompressLaunch& a);
int64_t launch_compress_split_96(const CompressLaunch& a);
int64_t launch_compress_split_128(const CompressLaunch& a);
int64_t launch_compress_split_192(const CompressLaunch& a);
int64_t launch_compress_split_256(const CompressLaunch& a);
inline int64_t launch_compress_split(const CompressLaunch& a) {
    int64_t c = launch_compress_split_96(a);
    if (!c) c = launch_compress_split_128(a);
    if (!c) c = launch_compress_split_192(a);
    return c ? c : launch_compress_split_256(a);
}

}  // namespace deto
