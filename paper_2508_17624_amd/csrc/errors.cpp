// Thread-local error message and ABI version.
#include "ew_internal.h"

namespace {
thread_local char g_err[512] = "";
}

namespace ew {

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

void clear_error() { g_err[0] = '\0'; }

}  // namespace ew

extern "C" const char* ew_last_error(void) { return g_err; }
extern "C" int ew_abi_version(void) { return 4; }
