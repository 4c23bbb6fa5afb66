// Per-call plan blob (host side) and the launchers of the small bookkeeping and
// reduction kernels shared by the fused and the logits-given path.
#pragma once
#include <vector>

#include "common.h"

namespace adwin {

DevicePlan device_plan_at(unsigned char* ws_plan, int32_t B, int32_t* row_idx, int32_t* row_seq);

// large dynamic LDS of the row-resident logits kernel, once per device (logits_kernels.hip)
hipError_t logits_kernels_opt_in();
// looks up the current device's address of the library's static scratch array (logits_kernels.hip)
hipError_t logits_static_setup();

// --- launchers (all asynchronous on `st`) ---------------------------------------------
hipError_t launch_build_rows(const DevicePlan& pl, int32_t B, int64_t n_rows, int64_t n_pad,
                             hipStream_t st);
// copies `bytes` (a multiple of 16) of host memory to `dst`; the host bytes are taken
// before the call returns
hipError_t launch_upload(void* dst, const void* src_host, size_t bytes, hipStream_t st);
hipError_t launch_fill_f32(float* p, int64_t n, float v, hipStream_t st);
hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t st);

// Per-rollout sums of KL (and of ||g_t||^2 when `rownorm` is given) over the window and
// over the whole rollout; writes loss_prefix / loss_full.  seg is double [B][4].
hipError_t launch_segment_sums(const DevicePlan& pl, int32_t B, int probe, const float* klr,
                               const float* rownorm, double* seg, float* loss_prefix,
                               float* loss_full, hipStream_t st);

struct BatchArgs {
  DevicePlan pl;
  int32_t B;
  int32_t H;            // 0: no gradient statistics (logits-given path)
  int probe;
  int zero_grad;        // grad_scale == 0: every alignment is defined as 0
  const double* seg;    // [B][4]
  const float* up;      // [B][H] pooled prefix sums (unweighted)
  const float* uf;      // [B][H] pooled full-rollout sums
  double* racc;         // [B][4] scratch
  float* rho_pooled; float* rho_field; float* batch;
  int32_t* n_out; int64_t* n_adm_out; int64_t n_adm;
};
hipError_t launch_alignment_and_batch(const BatchArgs& a, hipStream_t st);

// Candidate-window audit (Sec. 4.2): alignment of the shared prefix window L_k, for every
// candidate k, with the full-rollout gradient, from the per-row gradients of one
// full-rollout pass.
struct CandArgs {
  DevicePlan pl;
  int32_t B, H, K;
  int reduction;
  int zero_grad;
  int32_t L[ADWIN_MAX_CANDIDATES];
  double inv_nadm[ADWIN_MAX_CANDIDATES];   // TOKEN_MEAN weight of candidate k: 1 / sum_i min(L_k, len_i)
  const float* g;        // [rows][H] per-row gradients, computed-row order (every row: probe mode)
  const float* pf;       // [chunks][H] column sums of g over kChunkRows-row chunks of each rollout
  const float* uf;       // [B][H] pooled full-rollout sums
  const float* rownorm;  // [rows] ||g_t||^2
  const double* seg;     // [B][4]; seg[4 i + 3] = sum of ||g_t||^2 over rollout i
  float* uc;             // [K][B][H] scratch: pooled prefix sums
  double* cacc;          // [K][B][4] scratch: rho pooled, valid, rho field, valid
  double* cS;            // [K][B]   scratch: sum of ||g_t||^2 over the prefix
  float* rho_pooled; float* rho_field; float* batch;   // outputs, may be NULL
};
hipError_t launch_candidate_audit(const CandArgs& a, hipStream_t st);

// Rollout-level summaries of per-row outputs (Sec. 3.1 top-k rejection; App. C loss
// distribution and prefix / suffix teacher log-probability).  Rows are packed positions;
// rollout i's computed positions are j < computed_i = (probe ? len_i : n_i).
struct SummaryArgs {
  DevicePlan pl;
  int32_t B, K;
  int probe;
  int32_t topk;
  int32_t L[ADWIN_MAX_CANDIDATES];
  const int32_t* t_rank;     // [T] or NULL
  const float* t_logp;       // [T] or NULL
  const float* kl;           // [T] or NULL
  double* acc;               // [B][kSummarySlots] scratch
  int32_t* first_reject;     // [B] or NULL (needs t_rank)
  float* logp_mean;          // [B + 1][2] or NULL (needs t_logp)
  float* loss_share;         // [K] or NULL (needs kl)
};
constexpr int kSummarySlots = ADWIN_MAX_CANDIDATES + 3;   // K candidate sums, total, logp prefix, logp suffix
hipError_t launch_summaries(const SummaryArgs& a, hipStream_t st);

// Cosine of two fp32 arrays of n elements into *out (0 if either norm is 0): fixed partition
// into kCosineBlocks contiguous pieces, double sums, pieces added in index order.
constexpr int kCosineBlocks = 1024;
hipError_t launch_cosine(const float* x, const float* y, int64_t n, double* partials /* [kCosineBlocks][3] */,
                         float* out, hipStream_t st);

// Optional per-phase timing with HIP events on the caller's stream (profiling entry
// points only).  begin()/end() bracket one launch; collect() waits and sums per phase.
class PhaseTimer {
 public:
  explicit PhaseTimer(hipStream_t st) : st_(st) {}
  ~PhaseTimer();
  // begin/end keep the first error they meet; collect returns it instead of times
  void begin(int phase);
  void end();
  hipError_t collect(float* phase_ms, int n_phases);
 private:
  struct Span { int phase; hipEvent_t a, b; };
  hipStream_t st_;
  std::vector<Span> spans_;
  hipError_t err_ = hipSuccess;
  bool open_ = false;
};

// RAII helper: no-op when the timer is null.
struct PhaseScope {
  PhaseTimer* t;
  PhaseScope(PhaseTimer* timer, int phase) : t(timer) { if (t) t->begin(phase); }
  ~PhaseScope() { if (t) t->end(); }
};

}  // namespace adwin
