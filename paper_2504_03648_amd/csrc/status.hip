// Version, status text and HIP error capture.
#include <cstring>

#include "common.h"

namespace aibx {

static thread_local char g_hip_error[256] = "";

int hip_failed(hipError_t e) {
  const char* s = hipGetErrorString(e);
  std::strncpy(g_hip_error, s ? s : "unknown HIP error", sizeof(g_hip_error) - 1);
  g_hip_error[sizeof(g_hip_error) - 1] = 0;
  return AIBX_ERR_HIP;
}

}  // namespace aibx

extern "C" {

int aibx_version(void) { return 200; }  // 0.2.0

int aibx_hash_version(void) { return 1; }

const char* aibx_strerror(int status) {
  switch (status) {
    case AIBX_OK: return "ok";
    case AIBX_ERR_INVALID_ARG: return "invalid argument";
    case AIBX_ERR_ALIGN: return "misaligned pointer, stride or size";
    case AIBX_ERR_UNSUPPORTED: return "unsupported configuration";
    case AIBX_ERR_HIP: return "HIP runtime error (see aibx_last_hip_error)";
    default: return "unknown status";
  }
}

const char* aibx_last_hip_error(void) { return aibx::g_hip_error; }

}  // extern "C"
