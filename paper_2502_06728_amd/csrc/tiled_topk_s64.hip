// Tiled top-k compress and indexed decompress, chunk size 64.
#define DETO_S 64
#ifdef DETO_TILED_ONLY_64_32   // development builds: one instantiation, seconds to compile
#define DETO_K_LIST(X) X(32)
#else
#define DETO_K_LIST(X) X(1) X(2) X(4) X(8) X(16) X(32)
#endif
#define DETO_COMPRESS_FN launch_compress_topk_s64
#define DETO_DECOMPRESS_FN launch_decompress_idx_s64
#include "tiled_topk_impl.hip.h"
