// Tiled top-k compress and indexed decompress with byte indices and bf16 or fp16 values at
// chunk size 32, the chunk size of the paper's experiments ("Overall Setup"), for the
// compression rates 1/2 ... 1/32.
#ifdef DETO_TILED_ONLY_64_32
#define DETO_NARROW_LIST(X)
#else
#define DETO_NARROW_LIST(X) X(32, 16) X(32, 8) X(32, 4) X(32, 2) X(32, 1)
#endif
#define DETO_COMPRESS_NARROW_FN launch_compress_topk_packed_s32
#define DETO_DECOMPRESS_NARROW_FN launch_decompress_idx_packed_s32
#include "tiled_narrow_impl.hip.h"
