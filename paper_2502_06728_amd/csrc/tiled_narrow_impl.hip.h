// Shared body of the narrow-payload translation units: instantiates the top-k compress and the
// indexed decompress kernels with byte indices and bf16 / fp16 values or two-bit signs for the
// (chunk, k) pairs in DETO_NARROW_LIST(X), and defines the two launchers named by
// DETO_COMPRESS_NARROW_FN / DETO_DECOMPRESS_NARROW_FN.  DETO_NARROW_TERNARY selects the sign
// payload (value format 3), otherwise the 16-bit formats (1 = bf16, 2 = fp16).
#include "tiled_kernels.hip.h"
#include "tiled_launch.h"

namespace deto {

namespace {
#ifdef DETO_NARROW_TERNARY
bool takes(int val_dtype) { return val_dtype == 3; }
#else
bool takes(int val_dtype) { return val_dtype == 1 || val_dtype == 2; }
#endif
}  // namespace

bool DETO_COMPRESS_NARROW_FN(const CompressLaunch& a) {
    if (!takes(a.p.val_dtype) || !a.p.idx_u8 || a.p.scheme != 0) return false;
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
#define LAUNCH(S, K, G, V)                                                                      \
    compress_tiled_topk<S, K, G, V><<<grid, kWave, 0, a.stream>>>(a.p, a.tiles, tail, a.grad,   \
                                                                  a.mom, a.idx, a.val, a.coeff_dbg)
#ifdef DETO_NARROW_TERNARY
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.grad_bf16) LAUNCH(S, K, true, 3); else LAUNCH(S, K, false, 3);                    \
        return true;                                                                            \
    }
#else
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.p.val_dtype == 1) {                                                               \
            if (a.grad_bf16) LAUNCH(S, K, true, 1); else LAUNCH(S, K, false, 1);                \
        } else {                                                                                \
            if (a.grad_bf16) LAUNCH(S, K, true, 2); else LAUNCH(S, K, false, 2);                \
        }                                                                                       \
        return true;                                                                            \
    }
#endif
    DETO_NARROW_LIST(X)
#undef X
#undef LAUNCH
    return false;
}

bool DETO_DECOMPRESS_NARROW_FN(const DecompressLaunch& a) {
    if (!takes(a.p.val_dtype) || !a.p.idx_u8 || !a.idx || a.p.adam) return false;
    const unsigned grid = tiled_grid(a.tiles, a.n_chunks);
    const TailRange tail{a.n, a.n_chunks};
#define LAUNCH(S, K, B, V)                                                                      \
    decompress_tiled<S, K, B, V><<<grid, kWave, 0, a.stream>>>(                                 \
        a.p, a.tiles, tail, a.idx, a.idx_stride, a.val, a.val_stride, a.params,                 \
        AdamPtrs{nullptr, nullptr, nullptr}, a.presign_dbg)
#ifdef DETO_NARROW_TERNARY
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.param_bf16) LAUNCH(S, K, true, 3); else LAUNCH(S, K, false, 3);                   \
        return true;                                                                            \
    }
#else
#define X(S, K)                                                                                 \
    if (a.p.s == S && a.p.k == K) {                                                             \
        if (a.p.val_dtype == 1) {                                                               \
            if (a.param_bf16) LAUNCH(S, K, true, 1); else LAUNCH(S, K, false, 1);               \
        } else {                                                                                \
            if (a.param_bf16) LAUNCH(S, K, true, 2); else LAUNCH(S, K, false, 2);               \
        }                                                                                       \
        return true;                                                                            \
    }
#endif
    DETO_NARROW_LIST(X)
#undef X
#undef LAUNCH
    return false;
}

}  // namespace deto
