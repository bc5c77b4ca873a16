// Striding / Random with a narrow payload at chunk size 32, rates 1/2 ... 1/32: the setting of
// the paper's experiments (chunk size 32, only signs synchronised, "Overall Setup").
#ifdef DETO_TILED_ONLY_64_32
#define DETO_SCHEME_NARROW_LIST(X)
#else
#define DETO_SCHEME_NARROW_LIST(X) X(32, 16) X(32, 8) X(32, 4) X(32, 2) X(32, 1)
#endif
#define DETO_COMPRESS_SCHEME_NARROW_FN launch_compress_scheme_narrow_s32
#define DETO_DECOMPRESS_SCHEME_NARROW_FN launch_decompress_scheme_narrow_s32
#include "tiled_scheme_narrow_impl.hip.h"
