// Status strings and per-thread HIP error text.
#include <stdio.h>
#include "common.h"

namespace dat {
static thread_local char g_err[512] = "";

dat_status hip_fail(hipError_t e, const char* what, const char* file, int line) {
  snprintf(g_err, sizeof(g_err), "%s (%d) from %s at %s:%d", hipGetErrorString(e), (int)e, what, file, line);
  return DAT_ERR_HIP;
}

// Records a message of the library's own for dat_last_error() and returns `status`.
dat_status fail_with(dat_status status, const char* text) {
  snprintf(g_err, sizeof(g_err), "%s", text);
  return status;
}
}  // namespace dat

extern "C" const char* dat_last_error(void) { return dat::g_err; }

extern "C" const char* dat_status_string(dat_status s) {
  switch (s) {
    case DAT_OK: return "ok";
    case DAT_ERR_ARG: return "invalid argument";
    case DAT_ERR_SHAPE: return "shape not supported by this model";
    case DAT_ERR_NOMEM: return "out of memory";
    case DAT_ERR_NONFINITE: return "non-finite value";
    case DAT_ERR_HIP: return "HIP runtime error";
    case DAT_ERR_UNSUPPORTED: return "unsupported";
  }
  return "unknown status";
}
