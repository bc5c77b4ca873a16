// Tiled indexed decompress with Decoupled AdamW as the underlying optimizer (chunk sizes 64
// and 32, the paper's default).
#include "tiled_kernels.hip.h"
#include "tiled_launch.h"

#ifdef DETO_TILED_ONLY_64_32
#define DETO_ADAMW_LIST(X) X(64, 32)
#else
#define DETO_ADAMW_LIST(X) X(64, 32) X(64, 16) X(64, 8) X(32, 16) X(32, 8) X(32, 4) X(32, 2)
#endif

namespace deto {

bool launch_decompress_adamw(const DecompressLaunch& a) {
    if (!a.p.adam || !a.idx || a.p.val_dtype != 0 || a.p.idx_u8) return false;
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.param_bf16)                                                                       \
            decompress_tiled<S, K, true, 0, true><<<grid, kWave, 0, a.stream>>>(                \
                a.p, a.tiles, tail, a.idx, a.idx_stride, a.val, a.val_stride, a.params, a.adam,       \
                a.presign_dbg);                                                                 \
        else                                                                                    \
            decompress_tiled<S, K, false, 0, true><<<grid, kWave, 0, a.stream>>>(               \
                a.p, a.tiles, tail, a.idx, a.idx_stride, a.val, a.val_stride, a.params, a.adam,       \
                a.presign_dbg);                                                                 \
        return true;                                                                            \
    }
    DETO_ADAMW_LIST(X)
#undef X
    return false;
}

// Striding / Random (no transmitted indices) with Decoupled AdamW
#ifdef DETO_TILED_ONLY_64_32
#define DETO_ADAMW_SCHEME_LIST(X) X(64, 32)
#else
#define DETO_ADAMW_SCHEME_LIST(X) X(64, 32) X(64, 16) X(64, 8) X(32, 16) X(32, 8) X(32, 4) X(32, 2)
#endif

bool launch_decompress_scheme_adamw(const DecompressLaunch& a) {
    if (!a.p.adam || a.idx || a.p.val_dtype != 0) return false;
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
    const MaskWords mw{{a.stride_mask[0], a.stride_mask[1], a.stride_mask[2], a.stride_mask[3]}};
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.param_bf16)                                                                       \
            decompress_tiled_scheme<S, K, true, true><<<grid, kWave, 0, a.stream>>>(            \
                a.p, mw, a.tiles, tail, static_cast<const float*>(a.val), a.val_stride, a.params, \
                a.adam, a.presign_dbg);                                                         \
        else                                                                                    \
            decompress_tiled_scheme<S, K, false, true><<<grid, kWave, 0, a.stream>>>(           \
                a.p, mw, a.tiles, tail, static_cast<const float*>(a.val), a.val_stride, a.params, \
                a.adam, a.presign_dbg);                                                         \
        return true;                                                                            \
    }
    DETO_ADAMW_SCHEME_LIST(X)
#undef X
    return false;
}

}  // namespace deto
