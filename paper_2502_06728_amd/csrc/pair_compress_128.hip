// Two-lanes-per-chunk compress kernels (chunk size 128; any k; top-k selection).
#include "pair_kernels.hip.h"
#include "tiled_launch.h"

#ifdef DETO_TILED_ONLY_64_32
#define DETO_PAIR_ONE(X)
#else
#define DETO_PAIR_ONE(X) X(128)
#endif

namespace deto {

int64_t launch_compress_pair_128(const CompressLaunch& a) {
    const KParams& p = a.p;
    if (p.scheme != 0 || !p.use_dct || p.val_dtype == 3) return 0;
    const int64_t tiles = (a.n / p.s) / kMfmaChunks;
    // one workgroup per tile plus one per chunk past the last full tile
    const int64_t grid64 = tiles + (a.n_chunks - tiles * kMfmaChunks);
    if (tiles <= 0 || grid64 > 0x7FFFFFFF) return 0;
#define X(S)                                                                                    \
    if (p.s == S) {                                                                             \
        const unsigned grid = static_cast<unsigned>(grid64);                                        \
        if (a.grad_bf16)                                                                        \
            compress_pair<S, true><<<grid, kWave, 0, a.stream>>>(                               \
                p, tiles, a.n, a.n_chunks, a.grad, a.mom, a.idx, a.val, a.coeff_dbg);           \
        else                                                                                    \
            compress_pair<S, false><<<grid, kWave, 0, a.stream>>>(                              \
                p, tiles, a.n, a.n_chunks, a.grad, a.mom, a.idx, a.val, a.coeff_dbg);           \
        return a.n_chunks;   /* the tail chunks ride along */                                   \
    }
    DETO_PAIR_ONE(X)
#undef X
    return 0;
}

}  // namespace deto
