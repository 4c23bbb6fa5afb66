// The little state the library keeps: per device, whether the kernel attributes have been set;
// per thread, the text of the last HIP error.
#include <atomic>
#include <cstdio>

#include "common.h"

namespace adwin {

static thread_local char g_hip_error[256] = "";

const char* last_hip_error_text() { return g_hip_error; }

void set_last_hip_error(hipError_t e, const char* where) {
  snprintf(g_hip_error, sizeof(g_hip_error), "HIP error %d (%s) at %s", (int)e,
           hipGetErrorString(e), where);
}

bool first_use_on_device(int slot) {
  static std::atomic<unsigned long long> seen[4];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63 || slot < 0 || slot > 3) return true;
  const unsigned long long bit = 1ull << dev;
  return (seen[slot].fetch_or(bit) & bit) == 0;
}

}  // namespace adwin
