// Error reporting shared by all entry points: a thread-local message, never an exception.
#include <cstdarg>
#include <cstdio>

#include "common.h"

namespace hctr {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

hctr_status fail(hctr_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

hctr_status check_hip(hipError_t e, const char* what) {
  if (e == hipSuccess) return HCTR_OK;
  snprintf(g_err, sizeof(g_err), "%s: %s", what, hipGetErrorString(e));
  return HCTR_E_DEVICE;
}

}  // namespace hctr

HCTR_API const char* hctr_last_error(void) { return hctr::g_err; }
