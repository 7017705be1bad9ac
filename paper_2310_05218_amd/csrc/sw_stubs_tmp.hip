#include "swconv_internal.h"
namespace swconv {
bool mfma_s8_supported(const Conv2dShape&) { return false; }
hipError_t launch_mfma_s8(const int8_t*, const int8_t*, int32_t*, const Conv2dShape&, hipStream_t) { return hipErrorInvalidValue; }
}
