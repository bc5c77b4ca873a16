// Shared body of tiled_scheme.hip / tiled_scheme_small.hip: instantiates the Striding / Random
// kernels (raw-momentum or coefficient domain) for the (chunk, k) pairs in DETO_SCHEME_LIST(X)
// and defines the two launchers named by DETO_COMPRESS_SCHEME_FN / DETO_DECOMPRESS_SCHEME_FN.
#include "tiled_kernels.hip.h"
#include "tiled_launch.h"

namespace deto {

namespace {
MaskWords words(const uint32_t (&w)[4]) { return MaskWords{{w[0], w[1], w[2], w[3]}}; }
}  // namespace

bool DETO_COMPRESS_SCHEME_FN(const CompressLaunch& a) {
    if (a.p.val_dtype != 0 || a.p.idx_u8) return false;   // fp32 values, int32 indices only
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.grad_bf16)                                                                        \
            compress_tiled_scheme<S, K, true><<<grid, kWave, 0, a.stream>>>(                    \
                a.p, words(a.stride_mask), a.tiles, tail, a.grad, a.mom, static_cast<int32_t*>(a.idx),        \
                static_cast<float*>(a.val), a.coeff_dbg);         \
        else                                                                                    \
            compress_tiled_scheme<S, K, false><<<grid, kWave, 0, a.stream>>>(                   \
                a.p, words(a.stride_mask), a.tiles, tail, a.grad, a.mom, static_cast<int32_t*>(a.idx),        \
                static_cast<float*>(a.val), a.coeff_dbg);         \
        return true;                                                                            \
    }
    DETO_SCHEME_LIST(X)
#undef X
    return false;
}

bool DETO_DECOMPRESS_SCHEME_FN(const DecompressLaunch& a) {
    if (a.idx || a.p.val_dtype != 0 || a.p.adam) return false;
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.param_bf16)                                                                       \
            decompress_tiled_scheme<S, K, true><<<grid, kWave, 0, a.stream>>>(                  \
                a.p, words(a.stride_mask), a.tiles, tail, static_cast<const float*>(a.val), a.val_stride,     \
                a.params, AdamPtrs{nullptr, nullptr, nullptr}, a.presign_dbg);     \
        else                                                                                    \
            decompress_tiled_scheme<S, K, false><<<grid, kWave, 0, a.stream>>>(                 \
                a.p, words(a.stride_mask), a.tiles, tail, static_cast<const float*>(a.val), a.val_stride,     \
                a.params, AdamPtrs{nullptr, nullptr, nullptr}, a.presign_dbg);     \
        return true;                                                                            \
    }
    DETO_SCHEME_LIST(X)
#undef X
    return false;
}

}  // namespace deto
