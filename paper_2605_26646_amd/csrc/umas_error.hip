// Thread-local error message of libumas.
#include "umas_common.h"

namespace umas {
namespace {
thread_local char g_msg[512] = "";
}

umas_status fail(umas_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_msg, sizeof(g_msg), fmt, ap);
  va_end(ap);
  return code;
}
}  // namespace umas

extern "C" const char* umas_last_error(void) { return umas::g_msg; }
