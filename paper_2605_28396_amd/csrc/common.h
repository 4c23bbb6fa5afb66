// Internal declarations shared by the translation units of libadwin_opd.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "adwin_opd.h"

namespace adwin {

constexpr int kTileTokens = 256;   // token rows per workgroup tile of the logit kernels
constexpr int kTileVocab  = 128;   // vocabulary rows per tile step of the logit kernels
constexpr int kBK         = 64;    // bf16 elements staged per k-step (128 B per row)
constexpr int kGradTile   = 256;   // rows and columns of one dZ*W_s output tile
constexpr int kChunkRows  = 128;   // rows per partial of the pooled-gradient reduction
constexpr int kMaxStrips  = 64;    // vocabulary strips of the statistics pass

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Result of the host planner (Sec. 4.1 bookkeeping) plus the launch geometry.
struct HostPlan {
  int64_t T = 0;
  int32_t B = 0;
  int64_t n_adm = 0;      // sum n_i
  int64_t n_rows = 0;     // rows actually computed: n_adm, or T in probe mode
  int64_t n_pad = 0;      // n_rows rounded up to a token tile
  int64_t n_chunks = 0;   // partials of the pooled reduction
};

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

int validate_ragged(int64_t T, int32_t B, const int64_t* offsets, const int32_t* window);

// True the first time it is called for (slot, current device): function attributes such as
// the dynamic-LDS opt-in are per device, so they are set once on every device that is used.
// `slot` distinguishes call sites (0..3).  Thread-safe.
bool first_use_on_device(int slot);

const char* last_hip_error_text();
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
