// Tiled top-k compress and indexed decompress with the narrow payload: byte indices and
// bf16 or fp16 values (chunk size 64).
#ifdef DETO_TILED_ONLY_64_32
#define DETO_NARROW_LIST(X) X(64, 32)
#else
#define DETO_NARROW_LIST(X) X(64, 32) X(64, 16) X(64, 8)
#endif
#define DETO_COMPRESS_NARROW_FN launch_compress_topk_packed
#define DETO_DECOMPRESS_NARROW_FN launch_decompress_idx_packed
#include "tiled_narrow_impl.hip.h"
