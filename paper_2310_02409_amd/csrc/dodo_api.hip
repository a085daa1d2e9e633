// Host-only entry points of libdodo: version, status text, nugget count.
#include <string.h>

#include "dodo_common.h"

namespace dodo {
static thread_local char g_hip_error_text[256] = "HIP runtime error";

int record_hip_error(hipError_t e) {
  const char* s = hipGetErrorString(e);
  strncpy(g_hip_error_text, s ? s : "unknown HIP error", sizeof(g_hip_error_text) - 1);
  g_hip_error_text[sizeof(g_hip_error_text) - 1] = '\0';
  return DODO_ERR_HIP;
}

int compute_units() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
  return cus;
}
}  // namespace dodo

extern "C" {

int dodo_version(void) { return DODO_VERSION; }

const char* dodo_status_string(int status) {
  switch (status) {
    case DODO_OK: return "ok";
    case DODO_ERR_INVALID_ARG: return "invalid argument";
    case DODO_ERR_UNSUPPORTED: return "unsupported dtype, head size or alignment";
    case DODO_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case DODO_ERR_HIP: return dodo::g_hip_error_text;
    case DODO_ERR_SCRATCH_LIMIT: return "problem exceeds the library's static scratch buffer";
    default: return "unknown status";
  }
}

// k = ceil(n / r), r = den/num (Sec. 2.3), with 1 <= k <= n (Eq. 7).
int64_t dodo_nugget_count(int64_t n, int64_t num, int64_t den) {
  if (num <= 0 || den <= 0) return -1;
  if (n <= 0) return 0;
  // n * num can exceed 63 bits only for absurd inputs; split to stay exact.
  const int64_t whole = n / den, rest = n % den;
  __int128 k = static_cast<__int128>(whole) * num + (static_cast<__int128>(rest) * num + den - 1) / den;
  if (k < 1) k = 1;
  if (k > n) k = n;
  return static_cast<int64_t>(k);
}

}  // extern "C"
