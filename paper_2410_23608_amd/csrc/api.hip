// Error reporting and version of libspa.
#include <cstdarg>
#include <cstdio>

#include "spa_common.h"

namespace spa {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SPA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return SPA_OK;
}

}  // namespace spa

extern "C" int spa_version(void) { return 100; }

extern "C" const char* spa_last_error(void) { return spa::g_err; }
