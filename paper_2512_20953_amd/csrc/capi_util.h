// Error reporting shared by the C ABI translation units.
#pragma once
#include <hip/hip_runtime.h>

namespace ah {
int set_error(int status, const char* fmt, ...);          // records the message, returns status
int hip_status(hipError_t e, const char* what);           // AH_OK or AH_EDEVICE with the HIP error text
}  // namespace ah
