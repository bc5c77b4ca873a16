// Two-lanes-per-chunk compress kernels (chunk size 192; any k; top-k selection).
#include "pair_kernels.hip.h"
#include "tiled_launch.h"

#ifdef DETO_TILED_ONLY_64_32
#define DETO_PAIR_ONE(X)
#else
#define DETO_PAIR_ONE(X) X(192)
#endif

namespace deto {

int64_t launch_compress_pair_192(const CompressLaunch& a) {
    const KParams& p = a.p;
    if (p.scheme != 0 || !p.use_dct || p.val_dtype == 3) return 0;
    const int64_t tiles = (a.n / p.s) / kMfmaChunks;
    if (tiles <= 0 || tiles > 0x7FFFFFFF) return 0;
#define X(S)                                                                                    \
    if (p.s == S) {                                                                             \
        const unsigned grid = static_cast<unsigned>(tiles);   /* one tile per workgroup */         \
        if (a.grad_bf16)                                                                        \
            compress_pair<S, true><<<grid, kWave, 0, a.stream>>>(p, tiles, a.grad, a.mom, a.idx,   \
                                                                 a.val, a.coeff_dbg);           \
        else                                                                                    \
            compress_pair<S, false><<<grid, kWave, 0, a.stream>>>(p, tiles, a.grad, a.mom, a.idx,  \
                                                                  a.val, a.coeff_dbg);          \
        return tiles * kMfmaChunks;                                                             \
    }
    DETO_PAIR_ONE(X)
#undef X
    return 0;
}

}  // namespace deto
