// Tiled top-k compress and indexed decompress, chunk size 128, k = 64 (one wavefront per
// SIMD: a chunk occupies 128 VGPRs of its lane).  One translation unit per k: these are the
// largest kernels of the library and compile side by side.
#define DETO_S 128
#ifdef DETO_TILED_ONLY_64_32
#define DETO_K_LIST(X)
#else
#define DETO_K_LIST(X) X(64)
#endif
#define DETO_COMPRESS_FN launch_compress_topk_s128_k64
#define DETO_DECOMPRESS_FN launch_decompress_idx_s128_k64
#include "tiled_topk_impl.hip.h"
