// Indexed decompress on 64-chunk tiles, chunk size 96 (Appendix B sweep): the fast DCT ends in
// 3-point transforms.  The compress half at this chunk size runs on the two-lanes-per-chunk
// kernels.
#define DETO_S 96
#ifdef DETO_TILED_ONLY_64_32
#define DETO_K_LIST(X)
#else
#define DETO_K_LIST(X) X(6) X(12) X(24) X(48)
#endif
#define DETO_DECOMPRESS_FN launch_decompress_idx_s96
#include "tiled_topk_impl.hip.h"
