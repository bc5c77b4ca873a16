// Tiled top-k compress and indexed decompress with the ternary payload: byte indices and the
// signs of the kept coefficients, two bits per entry.  Chunk size 64 at rates 1/2 and 1/4, and
// chunk size 32 at rates 1/2 ... 1/32: sign-only synchronisation at chunk size 32 is the
// configuration of the paper's experiments ("Overall Setup").
#define DETO_NARROW_TERNARY
#ifdef DETO_TILED_ONLY_64_32
#define DETO_NARROW_LIST(X) X(64, 32)
#else
#define DETO_NARROW_LIST(X) X(64, 32) X(64, 16) X(32, 16) X(32, 8) X(32, 4) X(32, 2) X(32, 1)
#endif
#define DETO_COMPRESS_NARROW_FN launch_compress_topk_ternary
#define DETO_DECOMPRESS_NARROW_FN launch_decompress_idx_ternary
#include "tiled_narrow_impl.hip.h"
