// Tiled top-k compress and indexed decompress, chunk size 16 (the smallest chunk of the
// paper's Appendix B sweep).
#define DETO_S 16
#ifdef DETO_TILED_ONLY_64_32
#define DETO_K_LIST(X)
#else
#define DETO_K_LIST(X) X(1) X(2) X(4) X(8)
#endif
#define DETO_COMPRESS_FN launch_compress_topk_s16
#define DETO_DECOMPRESS_FN launch_decompress_idx_s16
#include "tiled_topk_impl.hip.h"
