// Tiled Striding / Random kernels (compress, and decompress without transmitted indices):
// compression rates 1/2 ... 1/8 at chunk sizes 64 and 32.
#ifdef DETO_TILED_ONLY_64_32
#define DETO_SCHEME_LIST(X) X(64, 32)
#else
#define DETO_SCHEME_LIST(X) X(64, 32) X(64, 16) X(64, 8) X(32, 16) X(32, 8)
#endif
#define DETO_COMPRESS_SCHEME_FN launch_compress_scheme
#define DETO_DECOMPRESS_SCHEME_FN launch_decompress_scheme
#include "tiled_scheme_impl.hip.h"
