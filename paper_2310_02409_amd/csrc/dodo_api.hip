// Host-only entry points of libdodo: version, status text, nugget count.
#include <string.h>

#include <map>
#include <mutex>
#include <tuple>

#include "dodo_common.h"

namespace dodo {
static thread_local char g_hip_error_text[256] = "HIP runtime error";

int record_hip_error(hipError_t e) {
  const char* s = hipGetErrorString(e);
  strncpy(g_hip_error_text, s ? s : "unknown HIP error", sizeof(g_hip_error_text) - 1);
  g_hip_error_text[sizeof(g_hip_error_text) - 1] = '\0';
  return DODO_ERR_HIP;
}

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_cache_mutex;
int g_cus[kMaxDevices] = {};
std::map<std::tuple<int, const void*>, int> g_lds_granted;
std::map<std::tuple<int, const void*, int, size_t>, int> g_resident;

int current_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
  return dev;
}
}  // namespace

int compute_units() {
  const int dev = current_device();
  if (dev < 0) return 256;
  std::lock_guard<std::mutex> lock(g_cache_mutex);
  if (g_cus[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    g_cus[dev] = cus;
  }
  return g_cus[dev];
}

int allow_dynamic_lds(const void* kernel, int bytes) {
  const int dev = current_device();
  std::lock_guard<std::mutex> lock(g_cache_mutex);
  int& granted = g_lds_granted[std::make_tuple(dev, kernel)];
  if (bytes <= granted) return DODO_OK;
  DODO_HIP_TRY(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
  granted = bytes;
  return DODO_OK;
}

int resident_blocks_per_cu(const void* kernel, int threads, size_t lds, int fallback) {
  const int dev = current_device();
  std::lock_guard<std::mutex> lock(g_cache_mutex);
  int& n = g_resident[std::make_tuple(dev, kernel, threads, lds)];
  if (n == 0) {
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, lds) != hipSuccess || per_cu <= 0)
      per_cu = fallback;
    n = per_cu;
  }
  return n;
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
