// Tiled top-k compress and indexed decompress with the narrow payload: byte indices and
// bf16 or fp16 values (chunk size 64).
#include "tiled_kernels.hip.h"
#include "tiled_launch.h"

#ifdef DETO_TILED_ONLY_64_32
#define DETO_PACKED_LIST(X) X(64, 32)
#else
#define DETO_PACKED_LIST(X) X(64, 32) X(64, 16) X(64, 8)
#endif

namespace deto {

bool launch_compress_topk_packed(const CompressLaunch& a) {
    if ((a.p.val_dtype != 1 && a.p.val_dtype != 2) || !a.p.idx_u8 || a.p.scheme != 0) return false;
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
#define LAUNCH(S, K, G, V)                                                                      \
    compress_tiled_topk<S, K, G, V><<<grid, kWave, 0, a.stream>>>(a.p, a.tiles, tail, a.grad, a.mom,   \
                                                                  a.idx, a.val, a.coeff_dbg)
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.p.val_dtype == 1) {                                                               \
            if (a.grad_bf16) LAUNCH(S, K, true, 1); else LAUNCH(S, K, false, 1);                \
        } else {                                                                                \
            if (a.grad_bf16) LAUNCH(S, K, true, 2); else LAUNCH(S, K, false, 2);                \
        }                                                                                       \
        return true;                                                                            \
    }
    DETO_PACKED_LIST(X)
#undef X
#undef LAUNCH
    return false;
}

bool launch_decompress_idx_packed(const DecompressLaunch& a) {
    if ((a.p.val_dtype != 1 && a.p.val_dtype != 2) || !a.p.idx_u8 || !a.idx || a.p.adam)
        return false;
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
#define LAUNCH(S, K, B, V)                                                                      \
    decompress_tiled<S, K, B, V><<<grid, kWave, 0, a.stream>>>(                                 \
        a.p, a.tiles, tail, a.idx, a.idx_stride, a.val, a.val_stride, a.params,                       \
        AdamPtrs{nullptr, nullptr, nullptr}, a.presign_dbg)
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.p.val_dtype == 1) {                                                               \
            if (a.param_bf16) LAUNCH(S, K, true, 1); else LAUNCH(S, K, false, 1);               \
        } else {                                                                                \
            if (a.param_bf16) LAUNCH(S, K, true, 2); else LAUNCH(S, K, false, 2);               \
        }                                                                                       \
        return true;                                                                            \
    }
    DETO_PACKED_LIST(X)
#undef X
#undef LAUNCH
    return false;
}

}  // namespace deto
