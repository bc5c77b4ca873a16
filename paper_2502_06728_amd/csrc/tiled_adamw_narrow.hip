// Decompress with Decoupled AdamW as the underlying optimizer for the narrow payloads (byte
// indices with bf16 / fp16 values or two-bit signs; or no indices at all under Striding /
// Random).  Chunk size 32 at the rates 1/2 ... 1/32 -- the paper's experiments synchronise only
// signs at chunk size 32 ("Overall Setup") and run Decoupled AdamW on top -- and chunk size 64
// at rates 1/2 and 1/4.
#include "tiled_kernels.hip.h"
#include "tiled_launch.h"

#ifdef DETO_TILED_ONLY_64_32
#define DETO_ADAMW_NARROW_LIST(X) X(64, 32)
#else
#define DETO_ADAMW_NARROW_LIST(X) X(32, 16) X(32, 8) X(32, 4) X(32, 2) X(32, 1) X(64, 32) X(64, 16)
#endif

namespace deto {

namespace {

template <int S, int K, int V>
void indexed(const DecompressLaunch& a) {
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
    if (a.param_bf16)
        decompress_tiled<S, K, true, V, true><<<grid, kWave, 0, a.stream>>>(
            a.p, a.tiles, tail, a.idx, a.idx_stride, a.val, a.val_stride, a.params, a.adam,
            a.presign_dbg);
    else
        decompress_tiled<S, K, false, V, true><<<grid, kWave, 0, a.stream>>>(
            a.p, a.tiles, tail, a.idx, a.idx_stride, a.val, a.val_stride, a.params, a.adam,
            a.presign_dbg);
}

template <int S, int K, int V>
void values_only(const DecompressLaunch& a) {
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
    const MaskWords mw{{a.stride_mask[0], a.stride_mask[1], a.stride_mask[2], a.stride_mask[3]}};
    if (a.param_bf16)
        decompress_tiled_scheme<S, K, true, true, V><<<grid, kWave, 0, a.stream>>>(
            a.p, mw, a.tiles, tail, a.val, a.val_stride, a.params, a.adam, a.presign_dbg);
    else
        decompress_tiled_scheme<S, K, false, true, V><<<grid, kWave, 0, a.stream>>>(
            a.p, mw, a.tiles, tail, a.val, a.val_stride, a.params, a.adam, a.presign_dbg);
}

template <int S, int K, int V>
void one(const DecompressLaunch& a) {
    if (a.idx) indexed<S, K, V>(a);
    else values_only<S, K, V>(a);
}

}  // namespace

bool launch_decompress_adamw_narrow(const DecompressLaunch& a) {
    if (!a.p.adam || a.p.val_dtype < 1 || a.p.val_dtype > 3 || (a.idx && !a.p.idx_u8))
        return false;
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.p.val_dtype == 1) one<S, K, 1>(a);                                                \
        else if (a.p.val_dtype == 2) one<S, K, 2>(a);                                           \
        else one<S, K, 3>(a);                                                                   \
        return true;                                                                            \
    }
    DETO_ADAMW_NARROW_LIST(X)
#undef X
    return false;
}

}  // namespace deto
