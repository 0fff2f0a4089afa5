// Error reporting and version of the C ABI.
#include <string.h>

#include "hs_common.h"

namespace hs {
static thread_local char g_err[512] = "";

hs_status fail(hs_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}
void clear_error() { g_err[0] = 0; }
}  // namespace hs

extern "C" const char* hs_status_string(hs_status st) {
  switch (st) {
    case HS_OK: return "ok";
    case HS_ERR_NULL: return "a required pointer is NULL";
    case HS_ERR_SHAPE: return "invalid or inconsistent shape";
    case HS_ERR_UNSUPPORTED: return "unsupported configuration";
    case HS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case HS_ERR_RUNTIME: return "HIP runtime error";
  }
  return "unknown status";
}

extern "C" const char* hs_last_error(void) { return hs::g_err; }
extern "C" const char* hs_version(void) { return "0.1"; }
