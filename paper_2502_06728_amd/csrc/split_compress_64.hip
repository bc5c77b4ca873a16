// Lane-per-chunk, wavefront-per-coefficient-class compress kernels (chunk size 64: 2 classes;
// top-k selection, fp32 values + int32 indices, k <= 32), for small shards: two wavefronts
// share a tile, so a tile is done sooner than on the lane-per-chunk kernel, which wins on
// throughput once the launch is many occupancy rounds long.  Also for any k the lane-per-chunk
// kernel is not instantiated for, at every shard size.
#include "split_kernels.hip.h"
#include "tiled_launch.h"

namespace deto {

int64_t launch_compress_split_64(const CompressLaunch& a) {
    const KParams& p = a.p;
#ifdef DETO_TILED_ONLY_64_32
    return 0;
#else
    if (p.s != 64 || p.scheme != 0 || !p.use_dct || p.val_dtype != 0 || p.idx_u8 || p.k > 32)
        return 0;
    const int64_t tiles = (a.n / p.s) / kWave;
    // the lane-per-chunk kernels take k as a template argument: at any other k this kernel
    // serves every shard size
    const bool lane_per_chunk_has_k = p.k == 1 || p.k == 2 || p.k == 4 || p.k == 8 || p.k == 16 ||
                                      p.k == 32;
    if (tiles <= 0 || (lane_per_chunk_has_k && tiles > small_shard_tiles())) return 0;
    // one workgroup per full tile and one for the chunks left over (a partial tile)
    const int64_t grid64 = tiles + (a.n_chunks > tiles * kWave ? 1 : 0);
    if (grid64 > 0x7FFFFFFF) return 0;
    const unsigned grid = static_cast<unsigned>(grid64);
    constexpr int kThreads = SplitGeom<64, 2>::kThreads;
    int32_t* io = static_cast<int32_t*>(a.idx);
    float* vo = static_cast<float*>(a.val);
#define LAUNCH(BF16, TOP)                                                                  \
    compress_split<64, 2, BF16, TOP><<<grid, kThreads, 0, a.stream>>>(                  \
        p, tiles, a.n, a.n_chunks, a.grad, a.mom, io, vo, a.coeff_dbg)
    // a launch with k <= 16 sorts out only every lane's 16 largest magnitudes
    if (p.k <= 16) {
        if (a.grad_bf16) LAUNCH(true, 16);
        else LAUNCH(false, 16);
    } else {
        if (a.grad_bf16) LAUNCH(true, 0);
        else LAUNCH(false, 0);
    }
#undef LAUNCH
    return a.n_chunks;   // the tail chunks ride along
#endif
}

}  // namespace deto
