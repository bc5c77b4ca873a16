// Tiled Striding / Random kernels for the low compression rates of the paper's experiments
// (chunk size 32 with k down to 1, "Overall Setup"; 1/16 to 1/64 at chunk 64; chunk 16).
#ifdef DETO_TILED_ONLY_64_32
#define DETO_SCHEME_LIST(X)
#else
#define DETO_SCHEME_LIST(X) X(32, 4) X(32, 2) X(32, 1) X(64, 4) X(64, 2) X(64, 1) X(16, 2) X(16, 1)
#endif
#define DETO_COMPRESS_SCHEME_FN launch_compress_scheme_small
#define DETO_DECOMPRESS_SCHEME_FN launch_decompress_scheme_small
#include "tiled_scheme_impl.hip.h"
