// Error reporting of the C ABI.
#include "ll_common.h"

namespace ll {

static thread_local int g_last_hip_error = 0;

int hip_failed(hipError_t e) {
  g_last_hip_error = (int)e;
  (void)hipGetLastError();   // clear the sticky error so that later calls start clean
  return LL_EHIP;
}

}  // namespace ll

extern "C" {

const char* ll_error_string(int code) {
  switch (code) {
    case LL_OK: return "success";
    case LL_EINVAL: return "invalid argument (null pointer, bad size or alignment, k out of range, d not a multiple of 8)";
    case LL_EWORKSPACE: return "workspace missing, misaligned or smaller than required";
    case LL_EHIP: return "a HIP call failed (see ll_last_hip_error)";
    case LL_ESCRATCH: return "the shape needs more than the library's static scratch buffer holds (use ll_project with a workspace)";
    default: return "unknown error code";
  }
}

int ll_last_hip_error(void) { return ll::g_last_hip_error; }

}  // extern "C"
