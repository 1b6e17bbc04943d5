// Error reporting and version of libprobe.
#include <stdarg.h>
#include <string.h>

#include "common.hpp"

namespace probe {

static thread_local char g_last_error[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_last_error, sizeof g_last_error, fmt, ap);
  va_end(ap);
}

int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("%s: %s", what, hipGetErrorString(e));
    return PROBE_EHIP;
  }
  return PROBE_OK;
}

}  // namespace probe

extern "C" const char* probe_last_error_string(void) { return probe::g_last_error; }
extern "C" const char* probe_version(void) { return "0.1"; }
