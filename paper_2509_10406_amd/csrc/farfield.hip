// placeholder until the far-field stages land
#include "common.h"
size_t muse_farfield_ws_bytes(const MuseDims&, bool, int) { return 256; }
size_t muse_farfield_fixed_bytes(const MuseDims&, bool) { return 256; }
int muse_run_fwd(const MuseDims&, const void*, const void*, const void*, const float*, const int32_t*, const int32_t*,
                 void*, float*, int32_t*, int32_t*, void*, size_t, hipStream_t) { return MUSE_ERR_UNSUPPORTED; }
int muse_run_bwd(const MuseDims&, const void*, const void*, const void*, const void*, const float*, const void*,
                 const float*, const int32_t*, const int32_t*, const int32_t*, const int32_t*, void*, void*, void*,
                 void*, size_t, hipStream_t) { return MUSE_ERR_UNSUPPORTED; }
