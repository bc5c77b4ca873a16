// Striding / Random with a narrow payload at chunk size 64, rates 1/2 ... 1/16.
#ifdef DETO_TILED_ONLY_64_32
#define DETO_SCHEME_NARROW_LIST(X) X(64, 32)
#else
#define DETO_SCHEME_NARROW_LIST(X) X(64, 32) X(64, 16) X(64, 8) X(64, 4)
#endif
#define DETO_COMPRESS_SCHEME_NARROW_FN launch_compress_scheme_narrow_s64
#define DETO_DECOMPRESS_SCHEME_NARROW_FN launch_decompress_scheme_narrow_s64
#include "tiled_scheme_narrow_impl.hip.h"
