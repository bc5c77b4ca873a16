// Tiled top-k compress and indexed decompress, chunk size 32.
#define DETO_S 32
#ifdef DETO_TILED_ONLY_64_32
#define DETO_K_LIST(X)
#else
#define DETO_K_LIST(X) X(1) X(2) X(4) X(8) X(16)
#endif
#define DETO_COMPRESS_FN launch_compress_topk_s32
#define DETO_DECOMPRESS_FN launch_decompress_idx_s32
#include "tiled_topk_impl.hip.h"
