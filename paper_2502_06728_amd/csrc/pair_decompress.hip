// Two-lanes-per-chunk decompress-and-update kernels (chunk sizes 192 and 256; any k;
// transmitted indices; plain SGD update or Decoupled AdamW).
#include "pair_kernels.hip.h"
#include "tiled_launch.h"

namespace deto {

int64_t launch_decompress_pair(const DecompressLaunch& a) {
    const KParams& p = a.p;
    if (!a.idx || !p.use_dct || p.val_dtype == 3) return 0;
    const int64_t tiles = (a.n / p.s) / kMfmaChunks;
    // one workgroup per tile plus one per chunk past the last full tile
    const int64_t grid64 = tiles + (a.n_chunks - tiles * kMfmaChunks);
    if (tiles <= 0 || grid64 > 0x7FFFFFFF) return 0;
    // 16-byte payload loads: fp32 values, int32 indices, four entries never straddle a chunk
    // (the caller has checked the alignment of the bases and of the replica strides)
    const int vec = (p.val_dtype == 0 && !p.idx_u8 && p.k % 4 == 0) ? 1 : 0;
#define X(S)                                                                                    \
    if (p.s == S) {                                                                             \
        const unsigned grid = static_cast<unsigned>(grid64);                                        \
        if (a.param_bf16)                                                                       \
            decompress_pair<S, true><<<grid, kWave, 0, a.stream>>>(                             \
                p, tiles, a.n, a.n_chunks, vec, a.idx, a.idx_stride, a.val, a.val_stride, a.params, a.adam,      \
                a.presign_dbg);                                                                 \
        else                                                                                    \
            decompress_pair<S, false><<<grid, kWave, 0, a.stream>>>(                            \
                p, tiles, a.n, a.n_chunks, vec, a.idx, a.idx_stride, a.val, a.val_stride, a.params, a.adam,      \
                a.presign_dbg);                                                                 \
        return a.n_chunks;   /* the tail chunks ride along */                                   \
    }
    DETO_PAIR_S_LIST(X)
#undef X
    return 0;
}

}  // namespace deto
