// Lane-per-chunk, wavefront-per-coefficient-class decompress-and-update kernels (chunk sizes 192
// and 256: four classes; transmitted indices, fp32 values + int32 indices; plain SGD update or
// Decoupled AdamW).  Two classes at chunk 64, 96 and 128 for what the lane-per-chunk kernels of
// those sizes are not instantiated for (they take k as a template argument and do not include
// Decoupled AdamW above chunk 64): any k at run time, about a fifth slower than a lane per chunk,
// several times faster than the matrix-core and general kernels that served such shapes before.
#include "split_kernels.hip.h"
#include "tiled_launch.h"

namespace deto {

int64_t launch_decompress_split(const DecompressLaunch& a) {
    const KParams& p = a.p;
#ifdef DETO_TILED_ONLY_64_32
    return 0;
#else
    if (!a.idx || !p.use_dct || p.val_dtype != 0 || p.idx_u8) return 0;
    const int64_t tiles = (a.n / p.s) / kWave;
    // one workgroup per full tile and one for the chunks left over (a partial tile)
    const int64_t grid64 = tiles + (a.n_chunks > tiles * kWave ? 1 : 0);
    if (tiles <= 0 || grid64 > 0x7FFFFFFF) return 0;
    const unsigned grid = static_cast<unsigned>(grid64);
    const int32_t* idx = static_cast<const int32_t*>(a.idx);
    const float* val = static_cast<const float*>(a.val);
#define X(S, W)                                                                                 \
    if (p.s == S) {                                                                             \
        if (a.param_bf16)                                                                       \
            decompress_split<S, W, true><<<grid, W * kWave, 0, a.stream>>>(                     \
                p, tiles, a.n, a.n_chunks, idx, a.idx_stride, val, a.val_stride, a.params,     \
                a.adam, a.presign_dbg);                                                         \
        else                                                                                    \
            decompress_split<S, W, false><<<grid, W * kWave, 0, a.stream>>>(                    \
                p, tiles, a.n, a.n_chunks, idx, a.idx_stride, val, a.val_stride, a.params,     \
                a.adam, a.presign_dbg);                                                         \
        return a.n_chunks;   /* the tail chunks ride along */                                   \
    }
    X(192, 4) X(256, 4) X(64, 2) X(96, 2) X(128, 2)
#undef X
    return 0;
#endif
}

}  // namespace deto
