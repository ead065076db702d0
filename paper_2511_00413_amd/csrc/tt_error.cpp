#include "tt_internal.h"

namespace tt {
static thread_local char g_msg[512] = "";

tt_status fail(tt_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_msg, sizeof(g_msg), fmt, ap);
  va_end(ap);
  return code;
}
void clear_error() { g_msg[0] = '\0'; }
}  // namespace tt

extern "C" const char* tt_last_error(void) { return tt::g_msg; }
extern "C" int32_t tt_version(void) { return 100; }
