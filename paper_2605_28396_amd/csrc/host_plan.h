// Pure host declarations of libadwin_opd (no HIP header): tile constants, the planner of
// Sec. 4.1's integer bookkeeping and the layout of the plan blob it writes.  host_plan.cpp
// builds from this header alone, so that it can also be compiled with the host compiler's
// sanitizers and run on a machine without a GPU.
#pragma once
#include <stddef.h>
#include <stdint.h>
#include <vector>

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

// Byte offsets of the plan arrays inside one contiguous upload, a function of B only.
struct PlanBlobLayout {
  size_t o_offsets, o_comp_off, o_n, o_chunk_off, o_alpha_p, o_alpha_f, bytes;
  explicit PlanBlobLayout(int32_t B) {
    size_t o = 0;
    o_offsets = o;   o = align_up(o + sizeof(int64_t) * (size_t)(B + 1), 16);
    o_comp_off = o;  o = align_up(o + sizeof(int64_t) * (size_t)(B + 1), 16);
    o_n = o;         o = align_up(o + sizeof(int32_t) * (size_t)B, 16);
    o_chunk_off = o; o = align_up(o + sizeof(int32_t) * (size_t)(B + 1), 16);
    o_alpha_p = o;   o = align_up(o + sizeof(float) * (size_t)B, 16);
    o_alpha_f = o;   o = align_up(o + sizeof(float) * (size_t)B, 16);
    bytes = align_up(o, 256);
  }
};

int validate_ragged(int64_t T, int32_t B, const int64_t* offsets, const int32_t* window);

// Integer bookkeeping of Sec. 4.1 (n_i, first computed row and first reduction chunk of
// each rollout) and the per-rollout weights alpha^p_i, alpha^f_i of the chosen
// reduction.  `blob` may be NULL when only the counts are wanted.
HostPlan make_host_plan(int64_t T, int32_t B, const int64_t* offsets, const int32_t* window,
                        int probe, int reduction, std::vector<unsigned char>* blob);

// Text of the calling thread's last HIP error ("" if none); defined with the HIP-side state.
const char* last_hip_error_text();

}  // namespace adwin
