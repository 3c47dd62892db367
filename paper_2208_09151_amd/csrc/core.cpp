// Error reporting and version of the library (host only).
#include <cstdarg>
#include <cstdio>

#include "ginex.h"

namespace ginex {

static thread_local char g_error[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
}

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return code;
}

}  // namespace ginex

extern "C" const char* ginex_last_error(void) { return ginex::g_error; }
extern "C" int32_t ginex_version(void) { return 10100; }
