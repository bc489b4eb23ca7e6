// Backward of the expert-choice layer (derivative of Sec. 3.2, Eq. 2-4 with the
// TopK selection held constant).  Not built yet: the entry point validates its
// arguments and reports EC_ERR_UNSUPPORTED.
#include "ec_common.h"

namespace ecmoe {

size_t bwd_ws_bytes(int64_t, int64_t, int64_t, int64_t, int64_t, int) { return 0; }

int launch_backward(const void*, const void*, const void*, const void*, const void*, const float*, const float*,
                    const int32_t*, const void*, const void*, const void*, const void*, void*, float*, float*,
                    float*, int64_t, int64_t, int64_t, int64_t, int64_t, int, int, void*, const WsLayout&,
                    hipStream_t) {
    return EC_ERR_UNSUPPORTED;
}

}  // namespace ecmoe
