// Lane-per-chunk, wavefront-per-coefficient-class compress kernels (chunk size 128: 2 classes;
// top-k selection, fp32 values + int32 indices, k <= 64).
#include "split_kernels.hip.h"

#ifndef DETO_SPLIT_W
#define DETO_SPLIT_W 2
#endif
#include "tiled_launch.h"

namespace deto {

int64_t launch_compress_split_128(const CompressLaunch& a) {
    const KParams& p = a.p;
#ifdef DETO_TILED_ONLY_64_32
    return 0;
#else
    if (p.s != 128 || p.scheme != 0 || !p.use_dct || p.val_dtype != 0 || p.idx_u8 || p.k > 64)
        return 0;
    const int64_t tiles = (a.n / p.s) / kWave;
    // one workgroup per full tile and one for the chunks left over (a partial tile)
    const int64_t grid64 = tiles + (a.n_chunks > tiles * kWave ? 1 : 0);
    if (tiles <= 0 || grid64 > 0x7FFFFFFF) return 0;
    const unsigned grid = static_cast<unsigned>(grid64);
    constexpr int kThreads = SplitGeom<128, DETO_SPLIT_W>::kThreads;
    // a launch with k <= 16 sorts out only every lane's 16 largest magnitudes
    constexpr int kQ = SplitGeom<128, DETO_SPLIT_W>::Q;
    constexpr int kTop = (kQ % 16 == 0 && kQ > 16) ? 16 : 0;
    int32_t* io = static_cast<int32_t*>(a.idx);
    float* vo = static_cast<float*>(a.val);
#define LAUNCH(BF16, TOP)                                                                  \
    compress_split<128, DETO_SPLIT_W, BF16, TOP><<<grid, kThreads, 0, a.stream>>>(                 \
        p, tiles, a.n, a.n_chunks, a.grad, a.mom, io, vo, a.coeff_dbg)
    if (kTop > 0 && p.k <= kTop) {
        if (a.grad_bf16) LAUNCH(true, kTop);
        else LAUNCH(false, kTop);
    } else if (kQ % 32 == 0 && kQ > 32 && p.k <= 32) {
        // ... with k <= 32 the 32 largest
        if (a.grad_bf16) LAUNCH(true, 32);
        else LAUNCH(false, 32);
    } else {
        if (a.grad_bf16) LAUNCH(true, 0);
        else LAUNCH(false, 0);
    }
#undef LAUNCH
    return a.n_chunks;   // the tail chunks ride along
#endif
}

}  // namespace deto
