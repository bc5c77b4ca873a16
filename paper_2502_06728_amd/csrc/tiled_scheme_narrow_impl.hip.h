// Shared body of the translation units for Striding / Random with a narrow payload (bf16 or
// fp16 values, or two-bit signs; byte indices if the caller asks for indices at all):
// instantiates the kernels for the (chunk, k) pairs in DETO_SCHEME_NARROW_LIST(X) and defines
// the launchers named by DETO_COMPRESS_SCHEME_NARROW_FN / DETO_DECOMPRESS_SCHEME_NARROW_FN.
#include "tiled_kernels.hip.h"
#include "tiled_launch.h"

namespace deto {

namespace {

template <int S, int K, int V>
void compress_one(const CompressLaunch& a) {
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
    const MaskWords mw{{a.stride_mask[0], a.stride_mask[1], a.stride_mask[2], a.stride_mask[3]}};
    if (a.grad_bf16)
        compress_tiled_scheme<S, K, true, V><<<grid, kWave, 0, a.stream>>>(
            a.p, mw, a.tiles, tail, a.grad, a.mom, a.idx, a.val, a.coeff_dbg);
    else
        compress_tiled_scheme<S, K, false, V><<<grid, kWave, 0, a.stream>>>(
            a.p, mw, a.tiles, tail, a.grad, a.mom, a.idx, a.val, a.coeff_dbg);
}

template <int S, int K, int V>
void decompress_one(const DecompressLaunch& a) {
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
    const MaskWords mw{{a.stride_mask[0], a.stride_mask[1], a.stride_mask[2], a.stride_mask[3]}};
    if (a.param_bf16)
        decompress_tiled_scheme<S, K, true, false, V><<<grid, kWave, 0, a.stream>>>(
            a.p, mw, a.tiles, tail, a.val, a.val_stride, a.params,
            AdamPtrs{nullptr, nullptr, nullptr}, a.presign_dbg);
    else
        decompress_tiled_scheme<S, K, false, false, V><<<grid, kWave, 0, a.stream>>>(
            a.p, mw, a.tiles, tail, a.val, a.val_stride, a.params,
            AdamPtrs{nullptr, nullptr, nullptr}, a.presign_dbg);
}

}  // namespace

bool DETO_COMPRESS_SCHEME_NARROW_FN(const CompressLaunch& a) {
    // indices, if wanted, leave as bytes
    if (a.p.scheme == 0 || a.p.val_dtype < 1 || a.p.val_dtype > 3 || (a.idx && !a.p.idx_u8))
        return false;
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.p.val_dtype == 1) compress_one<S, K, 1>(a);                                       \
        else if (a.p.val_dtype == 2) compress_one<S, K, 2>(a);                                  \
        else compress_one<S, K, 3>(a);                                                          \
        return true;                                                                            \
    }
    DETO_SCHEME_NARROW_LIST(X)
#undef X
    return false;
}

bool DETO_DECOMPRESS_SCHEME_NARROW_FN(const DecompressLaunch& a) {
    if (a.idx || a.p.val_dtype < 1 || a.p.val_dtype > 3 || a.p.adam) return false;
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.p.val_dtype == 1) decompress_one<S, K, 1>(a);                                     \
        else if (a.p.val_dtype == 2) decompress_one<S, K, 2>(a);                                \
        else decompress_one<S, K, 3>(a);                                                        \
        return true;                                                                            \
    }
    DETO_SCHEME_NARROW_LIST(X)
#undef X
    return false;
}

}  // namespace deto
