// Internal declarations shared by the translation units of libadwin_opd.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "adwin_opd.h"
#include "host_plan.h"

namespace adwin {

// Device-resident plan, uploaded once per call (all arrays live in the workspace).
struct DevicePlan {
  const int64_t* offsets;    // [B+1]
  const int64_t* comp_off;   // [B+1] first computed-row index of each rollout
  const int32_t* n;          // [B]
  const int32_t* chunk_off;  // [B+1] first pooled-reduction chunk of each rollout
  const float* alpha_p;      // [B]
  const float* alpha_f;      // [B]
  int32_t* row_idx;          // [n_pad] packed row of each computed row (padded with a valid row)
  int32_t* row_seq;          // [n_pad] rollout of each computed row
};

// True the first time it is called for (slot, current device): function attributes such as
// the dynamic-LDS opt-in are per device, so they are set once on every device that is used.
// `slot` distinguishes call sites (0..3).  Thread-safe.
bool first_use_on_device(int slot);

void set_last_hip_error(hipError_t e, const char* where);

}  // namespace adwin

#define ADWIN_HIP_TRY(expr)                                   \
  do {                                                        \
    hipError_t e_ = (expr);                                   \
    if (e_ != hipSuccess) {                                   \
      ::adwin::set_last_hip_error(e_, #expr);                 \
      return ADWIN_E_HIP;                                     \
    }                                                         \
  } while (0)
