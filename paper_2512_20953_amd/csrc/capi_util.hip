#include "capi_util.h"
#include "ah_stage.h"
#include <cstdarg>
#include <cstdio>

namespace ah {
static thread_local char g_err[512] = "";
thread_local const char* g_where = "";

int set_error(int status, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return status;
}

int hip_status(hipError_t e, const char* what) {
  if (e == hipSuccess) return AH_OK;
  return set_error(AH_EDEVICE, "%s: %s (hipError %d) in %.200s", what, hipGetErrorString(e), (int)e, g_where);
}
}  // namespace ah

extern "C" const char* ah_last_error(void) { return ah::g_err; }
