// Tiled top-k compress and indexed decompress with the ternary payload: byte indices and the
// signs of the kept coefficients, two bits per entry (chunk size 64, k a multiple of 16).
#include "tiled_kernels.hip.h"
#include "tiled_launch.h"

#ifdef DETO_TILED_ONLY_64_32
#define DETO_TERNARY_LIST(X) X(64, 32)
#else
#define DETO_TERNARY_LIST(X) X(64, 32) X(64, 16)
#endif

namespace deto {

bool launch_compress_topk_ternary(const CompressLaunch& a) {
    if (a.p.val_dtype != 3 || !a.p.idx_u8 || a.p.scheme != 0) return false;
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.grad_bf16)                                                                        \
            compress_tiled_topk<S, K, true, 3><<<grid, kWave, 0, a.stream>>>(                   \
                a.p, a.tiles, tail, a.grad, a.mom, a.idx, a.val, a.coeff_dbg);                  \
        else                                                                                    \
            compress_tiled_topk<S, K, false, 3><<<grid, kWave, 0, a.stream>>>(                  \
                a.p, a.tiles, tail, a.grad, a.mom, a.idx, a.val, a.coeff_dbg);                  \
        return true;                                                                            \
    }
    DETO_TERNARY_LIST(X)
#undef X
    return false;
}

bool launch_decompress_idx_ternary(const DecompressLaunch& a) {
    if (a.p.val_dtype != 3 || !a.p.idx_u8 || !a.idx || a.p.adam) return false;
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.param_bf16)                                                                       \
            decompress_tiled<S, K, true, 3><<<grid, kWave, 0, a.stream>>>(                      \
                a.p, a.tiles, tail, a.idx, a.idx_stride, a.val, a.val_stride, a.params,         \
                AdamPtrs{nullptr, nullptr, nullptr}, a.presign_dbg);                            \
        else                                                                                    \
            decompress_tiled<S, K, false, 3><<<grid, kWave, 0, a.stream>>>(                     \
                a.p, a.tiles, tail, a.idx, a.idx_stride, a.val, a.val_stride, a.params,         \
                AdamPtrs{nullptr, nullptr, nullptr}, a.presign_dbg);                            \
        return true;                                                                            \
    }
    DETO_TERNARY_LIST(X)
#undef X
    return false;
}

}  // namespace deto
