// Shared between the translation units of the fused path: tile geometry, the argument
// blocks of its kernels and the host-side launchers.  The kernels live in
// sweep_kernels.hip (LM-head projections, row statistics, gradient factors) and
// grad_kernels.hip (combine pass, gradient contractions, scale + scatter); fused_host.hip
// lays out the workspace and strings the launches together.
#ifndef ADWIN_FUSED_SHARED_H
#define ADWIN_FUSED_SHARED_H

#include "device_utils.h"
#include "plan_device.h"

namespace adwin {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kRowBytes = kBK * 2;   // 128 B of k per staged row

// Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
// virtual ids so that the tiles sharing operands also share an L2.
__device__ __forceinline__ int xcd_contiguous_id(int bid, int nb) {
  const int xcd = bid & 7, loc = bid >> 3;
  const int base = nb >> 3, rem = nb & 7;
  return xcd * base + (xcd < rem ? xcd : rem) + loc;
}

// One wave instruction of a direct global->LDS load: lane l moves the 16 bytes at
// sbase + voff(l) to LDS address lds_base + IMM + 16 l (M0 = LDS destination of the wave;
// scalar base + 32-bit lane offset).  Such loads return in order and are waited for with an
// explicit s_waitcnt vmcnt(N).  The destination is given as scalar base + literal and added
// straight into M0, and the callers keep the wave's share of both addresses in operands that
// are set up once, so that a load costs three instructions: a wave issues one instruction at a
// time and the loads share the shadow of an MFMA with LDS reads.
template <int IMM>
__device__ __forceinline__ void dma16_at(uint32_t lds_base, uint32_t voff, const char* sbase) {
  asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_base), "v"(voff), "s"(sbase), "n"(IMM) : "memory", "scc");
}

// Wave-uniform bookkeeping of a k-step pipeline, written as instructions at a fixed place:
// plain scalar arithmetic has no place of its own in the pinned instruction order of a k-step
// and would be gathered in front of the k-step's first MFMA, where the wave, which issues one
// instruction at a time, keeps the matrix pipe waiting.
// Ring slot after slot x (LDS addresses; the ring is [begin, end), slots STEP bytes apart).
template <int STEP>
__device__ __forceinline__ uint32_t ring_next(uint32_t x, uint32_t ring_begin, uint32_t ring_end) {
  uint32_t y;
  asm volatile("s_add_u32 %0, %1, %4\n\ts_cmp_lg_u32 %0, %2\n\ts_cselect_b32 %0, %0, %3"
               : "=&s"(y) : "s"(x), "s"(ring_end), "s"(ring_begin), "n"(STEP) : "scc");
  return y;
}
// 64-bit address, kept as two halves, += BYTES.
template <int BYTES>
__device__ __forceinline__ void addr_advance(uint32_t& lo, uint32_t& hi) {
  asm volatile("s_add_u32 %0, %0, %2\n\ts_addc_u32 %1, %1, 0" : "+s"(lo), "+s"(hi) : "n"(BYTES) : "scc");
}
__device__ __forceinline__ const char* addr_of(uint32_t lo, uint32_t hi) {
  return (const char*)(((uint64_t)hi << 32) | lo);
}

// a fragment (8 bf16 of one row) in the LDS, addressed by its 32-bit LDS address
typedef const __attribute__((address_space(3))) bf16x8* LdsFragPtr;
__device__ __forceinline__ LdsFragPtr lds_frag(uint32_t addr) { return (LdsFragPtr)(uintptr_t)addr; }

template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// Slab layout (the A operand of the gradient GEMM, see "Tile images" below): block
// (row tile, k-step) of 256 rows x 64 vocabulary entries, row r at r * 64 elements, its
// 8-entry chunk c at chunk position c ^ ((r >> 1) & 7).  A 256 x 128 logit tile covers the
// two consecutive blocks 2 vt and 2 vt + 1 of its row tile; `blk` points at the first.
constexpr int kSlabBlock = kTileTokens * kBK;   // elements per block
constexpr int kImgBytesSlab = kSlabBlock * 2;   // 32 KiB

// Blocks of the gradient GEMM's operand images: 256 rows x 64 k-entries (see grad_kernels.hip).
constexpr int kImgElems = kGradTile * kBK;            // bf16 elements per block
constexpr int kImgBytes = kImgElems * 2;              // 32 KiB

// Heavy entries.  The logit gradient dz = p_s ((z_s - z_t) - mu) is contracted with W_s as
// bf16.  On a peaked row a handful of entries carry the whole gradient row and their rounding
// (2^-9 relative each) does not average out, so every entry with p_s >= kHeavyP is taken out
// of the bf16 operand (stored as an exact zero) and listed per computed row instead; the
// scale-and-scatter kernel recomputes those few logits as fp32 dot products and adds
// dz W_s[v] in fp32.  Probabilities sum to 1, so a row has at most 1 / kHeavyP such entries;
// a flat row (the random-initialisation regime) has none.
constexpr float kHeavyP = 1.f / 32.f;
constexpr int kHeavySlots = 32;
struct HeavyList {
  int32_t* cnt;    // [n_pad] entries listed per computed row (zeroed at the start of a call)
  int32_t* v;      // [n_pad][kHeavySlots] vocabulary indices, in no particular order
};

// Lists entry v of computed row r; false when the row's list is full (the entry then stays in
// the bf16 operand).
__device__ __forceinline__ bool heavy_push(const HeavyList& hl, int64_t r, int v) {
  const int slot = atomicAdd(hl.cnt + r, 1);
  if (slot >= kHeavySlots) return false;
  hl.v[r * kHeavySlots + slot] = v;
  return true;
}

// x . y over H bf16 entries (H a multiple of 8), all 64 lanes of the wave; every lane gets the sum.
__device__ __forceinline__ float dot_bf16_row(const __bf16* x, const __bf16* y, int H, int lane) {
  float acc = 0.f;
  const uint4* px = (const uint4*)x;
  const uint4* py = (const uint4*)y;
  for (int q = lane; q < (H >> 3); q += 64) {
    const uint4 a = px[q], b = py[q];
    acc = fmaf(bf16_lo(a.x), bf16_lo(b.x), acc); acc = fmaf(bf16_hi(a.x), bf16_hi(b.x), acc);
    acc = fmaf(bf16_lo(a.y), bf16_lo(b.y), acc); acc = fmaf(bf16_hi(a.y), bf16_hi(b.y), acc);
    acc = fmaf(bf16_lo(a.z), bf16_lo(b.z), acc); acc = fmaf(bf16_hi(a.z), bf16_hi(b.z), acc);
    acc = fmaf(bf16_lo(a.w), bf16_lo(b.w), acc); acc = fmaf(bf16_hi(a.w), bf16_hi(b.w), acc);
  }
  return wave_sum(acc);
}

// ---------------------------------------------------------------------------------------
// Argument blocks
// ---------------------------------------------------------------------------------------
struct LogitPassArgs {
  const __bf16* h_s; const __bf16* h_t; const __bf16* W_s; const __bf16* W_t;
  int H_s, H_t, V;
  const int32_t* row_idx;      // [n_pad]
  int64_t n_pad;
  int tile0;                   // first token tile of this launch
  int n_tiles;                 // token tiles in this launch
  int strips;                  // vocabulary strips
  int tg;                      // token tiles per workgroup group (share W tiles in one L2)
  int vt_total;                // vocabulary tiles (of 128)
  // pass 1 out: [5][strips][n_pad]
  float* part;
  // pass 2 in / out
  const float* lse2; const float* mu;
  __bf16* slab; int64_t Vp;    // slab blocks of the launch's token tiles, tile0 first
  // single-sweep mode: fixed per-row references and the offset of the second slab half
  const float* ref_s2; const float* ref_t2; const float* mu0;
  int64_t e2_off;
  // per-(vocabulary tile, slab row) reference mu0 of the D factor, written by the sweep
  float* mu0t; int64_t mu0t_stride;
  // diagnostics mode: teacher logit of the sampled token and the token id (-1: none) per row
  const float* zy_t; const int32_t* yid;
  // direct-to-LDS kernel: tile images of the four operands (see row_image_kernel)
  const char* Wt_img; const char* Ws_img; const char* ht_img; const char* hs_img;
  HeavyList heavy;             // second sweep of the two-sweep scheme: entries taken out of dz
};

// Modes of the direct-to-LDS logit kernel.
constexpr int kModeStats = 0;   // online (running-max) statistics only
constexpr int kModeDz = 1;      // second sweep of the two-sweep scheme: dz tiles
constexpr int kModeSingle = 2;  // single sweep: fixed-reference statistics + D/E2 tiles
constexpr int kModeSingleDiag = 3;  // the same plus the teacher-side diagnostics of Sec. 3.1
constexpr int kModeSingleE2 = 4;      // single sweep that emits only the E2 factor (sampled estimator)
constexpr int kModeSingleE2Diag = 5;  // the same plus the diagnostics
constexpr int kModeSingleFwd = 6;     // single sweep, statistics only: nothing is written to the slab
constexpr int kModeSingleFwdDiag = 7; // the same plus the diagnostics

// Tile images of a row-major [rows, H] operand (see row_image_kernel).
struct RowImageArgs {
  const uint4* src; uint4* img; const int32_t* row_idx;
  int64_t n_rows; int H, nk, th;
  int permute;     // rows of every group of 32 in the order the logit kernels' epilogues want (W tiles)
};

// Merge of the strip partials into lse, mu, KL_t and c_t.
struct MergeArgs {
  const float* part; int strips; int64_t n_pad; int64_t n_rows;
  const int32_t* row_idx;
  const __bf16* h_s; const __bf16* h_t; const __bf16* W_s; const __bf16* W_t;
  int H_s, H_t, V;
  const int32_t* ids;
  float* lse2; float* mu; float* klr;
  float* lse_s;                // [n_pad] student log-sum-exp in nats (for the heavy entries)
  float* alive;                // [n_pad] two-sweep merge: 1, or 0 for an excluded (non-finite) row
  float* kl; float* c;
  uint32_t* status;
  // teacher-side diagnostics (single-sweep merge only); part planes 3 and 4 hold
  // sum e_t z_t and the rank count when `diag` is set
  int diag;
  float* t_logp; float* t_entropy; int32_t* t_rank;
  float* cr;     // [n_pad] c_t per computed row, for the sampled estimator (else NULL)
};

struct MergeSingleArgs {
  MergeArgs m;                 // part: [3][strips][n_pad] sums Z_s, A, Z_t
  const float* ref_s2; const float* ref_t2;
  float* mu_out; float* inv_z;
  int64_t row0, rows;          // computed rows [row0, row0 + rows) of this launch (one slab)
};

// Logits of the sampled token under both models (see token_logit_kernel).
struct TokenLogitArgs {
  const int32_t* row_idx; const int32_t* ids;
  const __bf16* h_s; const __bf16* W_s; const __bf16* h_t; const __bf16* W_t;
  int H_s, H_t, V;
  int64_t n_pad;
  float* zy_s; float* zy_t; int32_t* yid;
};

// Combine pass over one slab (see combine_kernel).
struct CombineArgs {
  uint4* slab; int64_t e2_vec;          // E2 lies e2_vec 16-byte vectors after D
  const float* mu; const float* inv_z;      // per computed row
  const float* mu0t; int64_t mu0t_stride;   // reference of D per (vocabulary tile, slab row)
  int64_t row0;                         // computed-row index of slab row 0
  int nk;                               // k-steps (blocks) per row tile
  // TR: also the transpose of w * dz as tile images for the head-weight GEMMs (rows =
  // vocabulary entries in tiles of 256, k = slab rows): block (vt, kr) with kr = 4 rt + j,
  // j = 0..3.  w = grad_scale * alpha of the row under the prefix objective (dzT_p; 0 outside
  // the window) and under the full-rollout objective (dzT_f); the weight is applied in fp32
  // before the one rounding to bf16.  Either image may be NULL.
  uint4* dzT_p; uint4* dzT_f; int nkr;  // k-steps (of 64 slab rows) per vocabulary tile
  DevicePlan pl; int64_t n_rows; float grad_scale;
  // SAMPLED (with TR): the slab holds only E2 and is left as it is; the transposed images take
  // Eq. 4's logit gradient c_t (e_{y_t} - p_s) = c_t (1[v = y_t] - E2 / Z_s), the one-hot term
  // entering before the rounding.  c_t and y_t per computed row (y_t = -1: none).
  const float* cr; const int32_t* yid;
  HeavyList heavy;             // entries with p_s >= kHeavyP leave the bf16 operand (expected estimator)
};

// Transposed h_s images of one slab (see hst_image_kernel).
struct HstImageArgs {
  const uint16_t* h_s; const int32_t* row_idx;
  int64_t row0;
  int H, nkr;
  uint16_t* img;
  const float* alive;     // per computed row; 0: excluded row, its column is written as zeros
};

// Gradient GEMM over tile images (see grad_gemm_kernel).
struct GradArgs {
  const __bf16* slab; const __bf16* WsT;   // tile images
  int nk_total;             // k-steps (blocks) per tile
  float* g;                 // [ksplit][g_rows][H]
  int64_t g_rows; int H;
  int64_t slab_row0;        // computed-row index of slab row 0
  int row_tiles, h_tiles, ksplit;
  int half_tiles;           // slab row tiles >= half_tiles hold the E2 factor: output rows
  int64_t half_off;         // half_off + slab_row0 + ... (single-sweep mode; else half_tiles = row_tiles)
  int64_t out_rows;         // rows of g that exist (rows at or beyond are not stored)
  int accumulate;           // add to g instead of overwriting it
};

// Scale + scatter of the row gradients (see finalize_kernel).
struct FinalizeArgs {
  DevicePlan pl; int B; int64_t T; int probe;
  float* g; int ksplit; int64_t n_pad; int H;
  int64_t g_rows;                          // rows per k-split plane of g
  const float* inv_z;                      // per computed row: 1 / Z_s (single sweep) or 1 (two sweeps);
                                           // 0 marks an excluded (non-finite) row: zeros everywhere
  // heavy entries: fp32 part of g, from the row's lse_s and mu and fresh dot products
  HeavyList heavy; const float* lse_s; const float* mu;
  const __bf16* h_s; const __bf16* h_t; const __bf16* W_t; int H_t;
  // sampled estimator (Eq. 4): g = c_t (W_s[y_t] - G2 inv_z), G2 = E2 W_s in the second half of
  // g; cr NULL: g is the contraction of the logit gradient itself, in the first half
  const float* cr; const int32_t* ids; const __bf16* W_s; int V;
  float grad_scale; int dh_bf16;
  void* dh_prefix; void* dh_full;
  float* rownorm;
};

// Pooled gradients per rollout (see pool_partial_kernel, pool_final_kernel).
struct PoolArgs {
  DevicePlan pl; int B; int probe; int H;
  const float* g; float* pp; float* pf;   // partials [n_chunks][H]
  float* up; float* uf;                   // [B][H]
};

// ---------------------------------------------------------------------------------------
// Launchers (asynchronous on `st`; the return value is that of the launch)
// ---------------------------------------------------------------------------------------
// sweep_kernels.hip
hipError_t sweep_kernels_opt_in();       // large dynamic LDS of the logit kernels, once per device
hipError_t launch_row_image(const RowImageArgs& a, unsigned tiles, hipStream_t st);
// mode: one of kMode*; dma false selects the register-staged kernel (kModeStats, kModeDz only)
hipError_t launch_logit_pass(int mode, bool dma, const LogitPassArgs& a, unsigned grid, hipStream_t st);
hipError_t launch_token_logit(const TokenLogitArgs& a, hipStream_t st);
hipError_t launch_make_refs(const float* part, int64_t n_pad, const float* zy_s, const float* zy_t,
                            const int32_t* yid, float* ref_s2, float* ref_t2, float* mu0, hipStream_t st);
hipError_t launch_merge_stats(const MergeArgs& a, hipStream_t st);
hipError_t launch_merge_single(const MergeSingleArgs& a, hipStream_t st);
// grad_kernels.hip
hipError_t grad_kernels_opt_in();
hipError_t launch_wst_image(const void* W_s, void* img, int V, int H, int nk, int h_tiles, hipStream_t st);
hipError_t launch_hst_image(const HstImageArgs& a, int h_tiles, hipStream_t st);
hipError_t launch_combine(bool transposed, bool sampled, const CombineArgs& a, int row_tiles, hipStream_t st);
hipError_t launch_grad_gemm(const GradArgs& a, hipStream_t st);
hipError_t launch_finalize(const FinalizeArgs& a, hipStream_t st);
hipError_t launch_pool_partial(const PoolArgs& a, int n_chunks, hipStream_t st);
hipError_t launch_pool_final(const PoolArgs& a, hipStream_t st);

}  // namespace adwin

#endif  // ADWIN_FUSED_SHARED_H
