// Error text and version of the C ABI.
#include <stdarg.h>
#include <stdio.h>

#include "../../include/rn50_hip.h"

namespace rn50 {
static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
void clear_error() { g_err[0] = 0; }
}  // namespace rn50

extern "C" const char* rn50_last_error(void) { return rn50::g_err; }
extern "C" int rn50_version(void) { return 1; }
