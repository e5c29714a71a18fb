// placeholder until the far-field backward lands
#include "ff_common.h"
int muse_run_bwd(const MuseDims&, const void*, const void*, const void*, const void*, const float*, const void*,
                 const float*, const int32_t*, const int32_t*, const int32_t*, const int32_t*, void*, void*, void*,
                 void*, size_t, hipStream_t) { return MUSE_ERR_UNSUPPORTED; }
