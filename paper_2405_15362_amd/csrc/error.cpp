// Thread-local error text behind pmc_last_error().
#include "pmc_internal.h"

namespace pmc {
namespace {
thread_local char g_error[512] = "";
}

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return code;
}
}  // namespace pmc

extern "C" const char* pmc_last_error(void) { return pmc::g_error; }
