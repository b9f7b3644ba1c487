// Error string and version of the C ABI.
#include <cstdarg>
#include <cstdio>

#include "../../include/augur.h"

namespace augur {

static thread_local char g_error[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
}

}  // namespace augur

extern "C" {
const char* augur_last_error(void) { return augur::g_error; }
const char* augur_version(void) { return "augur-gibbs-gfx950 0.1"; }
}
