// Shared body of the tiled_topk_s*.hip units: instantiates the top-k compress kernel and the
// indexed decompress kernel for chunk size DETO_S and the k values in DETO_K_LIST(X), and
// defines the two launchers named by DETO_COMPRESS_FN / DETO_DECOMPRESS_FN.  A unit that
// does not define DETO_COMPRESS_FN has the decompress kernel only (chunk sizes above 64).
#include "tiled_kernels.hip.h"
#include "tiled_launch.h"

namespace deto {

#ifdef DETO_COMPRESS_FN
bool DETO_COMPRESS_FN(const CompressLaunch& a) {
    if (a.p.s != DETO_S || a.p.val_dtype != 0 || a.p.idx_u8) return false;
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
#define X(K)                                                                                    \
    if (a.p.k == K) {                                                                           \
        if (a.grad_bf16)                                                                        \
            compress_tiled_topk<DETO_S, K, true><<<grid, kWave, 0, a.stream>>>(                 \
                a.p, a.tiles, tail, a.grad, a.mom, a.idx, a.val, a.coeff_dbg);                        \
        else                                                                                    \
            compress_tiled_topk<DETO_S, K, false><<<grid, kWave, 0, a.stream>>>(                \
                a.p, a.tiles, tail, a.grad, a.mom, a.idx, a.val, a.coeff_dbg);                        \
        return true;                                                                            \
    }
    DETO_K_LIST(X)
#undef X
    return false;
}
#endif

bool DETO_DECOMPRESS_FN(const DecompressLaunch& a) {
    if (a.p.s != DETO_S || !a.idx || a.p.val_dtype != 0 || a.p.idx_u8 || a.p.adam) return false;
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
#define X(K)                                                                                    \
    if (a.p.k == K) {                                                                           \
        if (a.param_bf16)                                                                       \
            decompress_tiled<DETO_S, K, true><<<grid, kWave, 0, a.stream>>>(                    \
                a.p, a.tiles, tail, a.idx, a.idx_stride, a.val, a.val_stride, a.params,               \
                AdamPtrs{nullptr, nullptr, nullptr}, a.presign_dbg);                                                                 \
        else                                                                                    \
            decompress_tiled<DETO_S, K, false><<<grid, kWave, 0, a.stream>>>(                   \
                a.p, a.tiles, tail, a.idx, a.idx_stride, a.val, a.val_stride, a.params,               \
                AdamPtrs{nullptr, nullptr, nullptr}, a.presign_dbg);                                                                 \
        return true;                                                                            \
    }
    DETO_K_LIST(X)
#undef X
    return false;
}

}  // namespace deto
