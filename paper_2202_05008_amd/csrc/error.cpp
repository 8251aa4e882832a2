// Thread-local error message and version string of the C ABI.
#include "common.h"

namespace evo {
static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
}  // namespace evo

extern "C" const char* evo_last_error(void) { return evo::g_err; }
extern "C" const char* evo_version(void) { return "evo-gfx950 0.1"; }
