// Indexed decompress on 64-chunk tiles, chunk size 128 (one wavefront per SIMD: a chunk
// occupies 128 VGPRs of its lane).  The compress half at this chunk size runs on the
// two-lanes-per-chunk kernels.
#define DETO_S 128
#ifdef DETO_TILED_ONLY_64_32
#define DETO_K_LIST(X)
#else
#define DETO_K_LIST(X) X(1) X(4) X(8) X(16) X(32) X(64)
#endif
#define DETO_DECOMPRESS_FN launch_decompress_idx_s128
#include "tiled_topk_impl.hip.h"
