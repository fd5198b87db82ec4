// 3-D scaling coordinates from the INT8 factors (placeholder until the kernels land).
#include "common.h"

extern "C" int rfx_mds3d(const int8_t*, const float*, int64_t, int32_t, int, int32_t, int32_t, float, const float*,
                         float*, float*, int32_t*, void*) {
    return rfx::fail(RFX_ERR_UNSUPPORTED, "rfx_mds3d: not implemented yet");
}
