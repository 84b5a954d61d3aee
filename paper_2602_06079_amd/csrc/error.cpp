// Thread-local error message behind canz_last_error(), and the version string.
#include <cstdio>

#include "canz.h"
#include "canz_internal.h"

namespace {
thread_local char g_msg[512] = "";
}

namespace canz {
int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_msg, sizeof(g_msg), fmt, ap);
  va_end(ap);
  return code;
}
}  // namespace canz

extern "C" const char* canz_last_error(void) { return g_msg; }
extern "C" const char* canz_version(void) { return "0.4.0"; }
