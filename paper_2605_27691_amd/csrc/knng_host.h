// Host-side helpers shared by the libknng translation units.
#pragma once
#include <hip/hip_runtime.h>

namespace knng {
// Remember the text of a failed HIP call (per thread) and return KNNG_EHIP.
int set_hip_error(hipError_t e, const char* what);
}  // namespace knng
