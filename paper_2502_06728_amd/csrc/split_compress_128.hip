// Lane-per-chunk, wavefront-per-coefficient-class compress kernels (chunk size 128: 2 classes,
// 4 on a small shard; top-k selection, fp32 values + int32 indices, k <= 64).
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
    int32_t* io = static_cast<int32_t*>(a.idx);
    float* vo = static_cast<float*>(a.val);
#define LAUNCH(W, BF16, TOP)                                                               \
    compress_split<128, W, BF16, TOP><<<grid, SplitGeom<128, W>::kThreads, 0, a.stream>>>( \
        p, tiles, a.n, a.n_chunks, a.grad, a.mom, io, vo, a.coeff_dbg)
    if (tiles <= small_shard_tiles()) {
        // a small shard: four classes (32 coefficients per lane, four wavefronts per tile)
        if (p.k <= 16) {
            if (a.grad_bf16) LAUNCH(4, true, 16);
            else LAUNCH(4, false, 16);
        } else {
            if (a.grad_bf16) LAUNCH(4, true, 0);
            else LAUNCH(4, false, 0);
        }
    } else if (p.k <= 16) {
        // a launch with k <= 16 sorts out only every lane's 16 largest magnitudes
        if (a.grad_bf16) LAUNCH(DETO_SPLIT_W, true, 16);
        else LAUNCH(DETO_SPLIT_W, false, 16);
    } else if (p.k <= 32) {
        // ... with k <= 32 the 32 largest
        if (a.grad_bf16) LAUNCH(DETO_SPLIT_W, true, 32);
        else LAUNCH(DETO_SPLIT_W, false, 32);
    } else {
        if (a.grad_bf16) LAUNCH(DETO_SPLIT_W, true, 0);
        else LAUNCH(DETO_SPLIT_W, false, 0);
    }
#undef LAUNCH
    return a.n_chunks;   // the tail chunks ride along
#endif
}

}  // namespace deto
