// Error reporting shared by the C ABI translation units.
#pragma once
#include <hip/hip_runtime.h>

namespace ah {
int set_error(int status, const char* fmt, ...);          // records the message, returns status
int hip_status(hipError_t e, const char* what);           // AH_OK or AH_EDEVICE with the HIP error text
// HIP keeps the last error of the calling thread until someone reads it.  The launch helpers
// check hipGetLastError() after each launch, so an entry point first discards whatever an
// earlier, unrelated runtime call of the host program left behind.
extern thread_local const char* g_where;                  // text of the HIP-calling expression last started
inline void discard_stale_hip_error() { (void)hipGetLastError(); }
}  // namespace ah
