// Matrix-core compress kernels (chunk sizes 32, 64, ..., 256; any k; top-k selection).
#include "mfma_kernels.hip.h"
#include "tiled_launch.h"

namespace deto {

int64_t launch_compress_mfma(const CompressLaunch& a) {
    const KParams& p = a.p;
    if (p.scheme != 0 || !p.use_dct || p.s % 32 != 0 || p.s > 256) return 0;
    if (p.val_dtype == 3) return 0;   // two-bit payload: general kernels
    const int64_t tiles = (a.n / p.s) / kMfmaChunks;
    if (tiles <= 0) return 0;
#define X(NB)                                                                                   \
    if (p.s == 32 * NB) {                                                                       \
        const unsigned grid = mfma_grid(tiles, MfmaGeom<NB>::kSmemBytes);                       \
        if (a.grad_bf16)                                                                        \
            compress_mfma<NB, true><<<grid, kWave, 0, a.stream>>>(p, tiles, a.grad, a.mom, a.idx,  \
                                                                  a.val, a.coeff_dbg);          \
        else                                                                                    \
            compress_mfma<NB, false><<<grid, kWave, 0, a.stream>>>(p, tiles, a.grad, a.mom, a.idx, \
                                                                   a.val, a.coeff_dbg);         \
        return tiles * kMfmaChunks;                                                             \
    }
    DETO_MFMA_NB_LIST(X)
#undef X
    return 0;
}

}  // namespace deto
