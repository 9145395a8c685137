// Thread-local last-error message behind dp_last_error().  Host code without any GPU call, so that the
// host-only parts of the library (partitioner, bubble filler, schedule search) also build on their own.
#include "../../include/dpipe.h"
#include "dp_errors.h"

#include <cstdarg>
#include <cstdio>

namespace dp {

static thread_local char g_err[512] = "";

int set_error(int code, const char* msg) {
  snprintf(g_err, sizeof(g_err), "%s", msg);
  return code;
}

int set_errorf(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

}  // namespace dp

extern "C" const char* dp_last_error(void) { return dp::g_err; }
