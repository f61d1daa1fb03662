#include "tl_internal.hpp"
namespace tl {
bool mfma_supports(int64_t, int64_t, int64_t) { return false; }
hipError_t launch_mfma(const __half*, const uint32_t*, float, __half*, int64_t, int64_t, int64_t,
                       hipStream_t) { return hipErrorNotSupported; }
}
