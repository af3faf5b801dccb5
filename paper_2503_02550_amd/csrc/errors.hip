// Thread-local error text behind sif_last_error().
#include <stdarg.h>
#include <stdio.h>
#include "launch.h"

namespace sif {

static thread_local char g_err[512] = "";

sif_status fail(sif_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

sif_status fail_hip(hipError_t e, const char* what) {
  return fail(SIF_E_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

sif_status check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail_hip(e, what);
  return SIF_OK;
}

}  // namespace sif

extern "C" const char* sif_last_error(void) { return sif::g_err; }
extern "C" int32_t sif_abi_version(void) { return 1; }
