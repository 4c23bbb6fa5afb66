// Fused path, second half: from the stored gradient factors to dL/dh_s and dL/dW_s.
//
// Combine  : once a slab's rows have their mu, the two factors the sweep stored collapse
//            in place into the logit gradient dz = p_s ((z_s - z_t) - mu) (Eq. 4 in
//            expectation, App. A.1); optionally also the transposed, weighted copies that
//            the head-weight contraction needs.
// GEMM     : g = dz W_s (and dW_s = (w dz)^T h_s) as bf16 MFMA GEMMs over tile images.
// Finalize : scale by grad_scale * alpha, scatter to dh_prefix / dh_full, row norms.
// Pool     : per-rollout column sums of g over the window and over the rollout (Sec. 4.2).
#include "fused_shared.h"
#include <utility>

namespace adwin {

// ---------------------------------------------------------------------------------------
// Tile images.  Both operands of the gradient GEMM live in memory as the exact LDS images
// of its k-steps: block (tile, kt) is 256 rows x 64 k-entries = 32 KiB, row r at r * 128 B,
// its 16-byte chunk c (k-entries 8 c .. 8 c + 7) at chunk position c ^ ((r >> 1) & 7).
// Blocks of one tile are consecutive in kt, so a workgroup streams each operand as one
// sequential run and every wave-load moves 1 KiB of consecutive bytes.
// ---------------------------------------------------------------------------------------

// element offset of (row r of the tile, k-entry k of the k-step) inside a block
__device__ __forceinline__ int img_elem(int r, int k) {
  return r * kBK + ((((k >> 3) ^ (r >> 1)) & 7) << 3) + (k & 7);
}

// W_s [V, H] -> images of W_s^T: tile = 256 hidden columns, k = vocabulary (zero beyond V).
// One workgroup per (k-step, hidden tile): reads 64 rows of W_s, writes one block.
__global__ __launch_bounds__(256) void wst_image_kernel(const uint16_t* __restrict__ W,
                                                        uint16_t* __restrict__ img, int V, int H,
                                                        int nk) {
  __shared__ uint16_t tile[kBK][kGradTile + 2];
  const int kt = blockIdx.x, ht = blockIdx.y;
  const int tid = threadIdx.x;
  for (int i = 0; i < kBK; ++i) {
    const int v = kt * kBK + i, h = ht * kGradTile + tid;
    tile[i][tid] = (v < V && h < H) ? W[(int64_t)v * H + h] : (uint16_t)0;
  }
  __syncthreads();
  uint16_t* blk = img + ((int64_t)ht * nk + kt) * kImgElems;
  // thread -> (row r, chunk position): 2048 chunks of 8 entries, 8 per thread
  for (int q = tid; q < kGradTile * 8; q += 256) {
    const int r = q >> 3, pos = q & 7, c = pos ^ ((r >> 1) & 7);
    uint16_t w[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) w[e] = tile[c * 8 + e][r];
    uint4 o;
    o.x = w[0] | ((uint32_t)w[1] << 16); o.y = w[2] | ((uint32_t)w[3] << 16);
    o.z = w[4] | ((uint32_t)w[5] << 16); o.w = w[6] | ((uint32_t)w[7] << 16);
    *(uint4*)(blk + q * 8) = o;
  }
}

// ---------------------------------------------------------------------------------------
// Combine.  Once a slab's rows have their mu (all strips merged), the two stored factors
// collapse into the logit gradient itself, dz = E2 (D - (mu - mu0)) / Z_s = p_s (d - mu),
// written over D in the same image order, and the gradient GEMM runs on one factor.  A
// streaming pass: 4 B read + 2 B written per slab element.
// ---------------------------------------------------------------------------------------

template <bool TR, bool SAMPLED = false>
__global__ __launch_bounds__(256) void combine_kernel(CombineArgs a) {
  // one workgroup per block (row tile rt = blockIdx.y, kt = blockIdx.x): 2048 vectors of 8
  // entries; vector q holds row q / 8, chunk position q % 8
  __shared__ __align__(16) uint16_t tile[TR ? kTileTokens : 1][TR ? kBK + 8 : 1];   // [row][entry], padded
  __shared__ float wrow[2][TR ? kTileTokens : 1];
  const int kt = blockIdx.x, rt = blockIdx.y;
  const int64_t blk = (int64_t)rt * a.nk + kt;
  uint4* p1 = a.slab + blk * (kImgBytesSlab / 16);
  const uint4* p2 = p1 + a.e2_vec;
  const int64_t rbase = a.row0 + (int64_t)rt * kTileTokens;
  if (TR) {
    const int64_t r = rbase + threadIdx.x;
    float wp = 0.f, wf = 0.f;
    if (r < a.n_rows && a.inv_z[r] != 0.f) {     // excluded rows carry weight 0
      const int i = a.pl.row_seq[r];
      wf = a.grad_scale * a.pl.alpha_f[i];
      wp = (r - a.pl.comp_off[i]) < a.pl.n[i] ? a.grad_scale * a.pl.alpha_p[i] : 0.f;
    }
    wrow[0][threadIdx.x] = wp;
    wrow[1][threadIdx.x] = wf;
    __syncthreads();
  }
  float dz[TR ? 8 : 1][8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int q = i * 256 + threadIdx.x;
    const int64_t r = rbase + (q >> 3);
    const float iz = a.inv_z[r];
    const uint4 y = p2[q];
    float d[8];
    if (SAMPLED) {
      const float c = a.cr[r], ciz = -c * iz;
      d[0] = bf16_lo(y.x) * ciz; d[1] = bf16_hi(y.x) * ciz; d[2] = bf16_lo(y.y) * ciz; d[3] = bf16_hi(y.y) * ciz;
      d[4] = bf16_lo(y.z) * ciz; d[5] = bf16_hi(y.z) * ciz; d[6] = bf16_lo(y.w) * ciz; d[7] = bf16_hi(y.w) * ciz;
      // entries of this vector: 64 kt + 8 (logical chunk) + e
      const int rl = q >> 3, v0 = kt * kBK + (((q & 7) ^ ((rl >> 1) & 7)) << 3);
      const int e_y = a.yid[r] - v0;
#pragma unroll
      for (int e = 0; e < 8; ++e) d[e] += (e == e_y) ? c : 0.f;
      if (TR) {
#pragma unroll
        for (int e = 0; e < 8; ++e) dz[i][e] = d[e];
      }
    } else {
      const float dl = a.mu[r] - a.mu0t[(int64_t)(kt >> 1) * a.mu0t_stride + rt * kTileTokens + (q >> 3)];
      const uint4 x = p1[q];
      float pv[8], xv[8];                      // p_s and the stored D of the vector's 8 entries
      pv[0] = bf16_lo(y.x) * iz; pv[1] = bf16_hi(y.x) * iz; pv[2] = bf16_lo(y.y) * iz; pv[3] = bf16_hi(y.y) * iz;
      pv[4] = bf16_lo(y.z) * iz; pv[5] = bf16_hi(y.z) * iz; pv[6] = bf16_lo(y.w) * iz; pv[7] = bf16_hi(y.w) * iz;
      xv[0] = bf16_lo(x.x); xv[1] = bf16_hi(x.x); xv[2] = bf16_lo(x.y); xv[3] = bf16_hi(x.y);
      xv[4] = bf16_lo(x.z); xv[5] = bf16_hi(x.z); xv[6] = bf16_lo(x.w); xv[7] = bf16_hi(x.w);
      const bool dead = iz == 0.f;             // excluded row: its factors may hold inf / NaN
      float pmax = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        d[e] = dead ? 0.f : (xv[e] - dl) * pv[e];
        pmax = fmaxf(pmax, pv[e]);
      }
      if (TR) {                                // the head-weight operand keeps every entry in bf16
#pragma unroll
        for (int e = 0; e < 8; ++e) dz[i][e] = d[e];
      }
      if (__builtin_expect(pmax >= kHeavyP && !dead, 0)) {
        // entries of this vector: 64 kt + 8 (logical chunk) + e
        const int rl = q >> 3, v0 = kt * kBK + (((q & 7) ^ ((rl >> 1) & 7)) << 3);
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (pv[e] >= kHeavyP && heavy_push(a.heavy, r, v0 + e)) d[e] = 0.f;
      }
      uint4 o;
      o.x = pack_bf16(d[0], d[1]); o.y = pack_bf16(d[2], d[3]);
      o.z = pack_bf16(d[4], d[5]); o.w = pack_bf16(d[6], d[7]);
      p1[q] = o;
    }
  }
  if (TR) {
    // this block's 64 entries are image rows (kt % 4) * 64 .. + 64 of vocabulary tile kt / 4;
    // its 256 slab rows are the k-steps 4 rt .. 4 rt + 3.  Vector u: k-step u / 512, image
    // row (u / 8) % 64, chunk position u % 8 -> one wave instruction writes 8 whole rows.
    const int vt = kt >> 2, row0 = (kt & 3) * kBK;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
      uint4* dst = which == 0 ? a.dzT_p : a.dzT_f;
      if (!dst) continue;
      __syncthreads();
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int q = i * 256 + threadIdx.x;
        const int rl = q >> 3;
        const float w = wrow[which][rl];
        const int c = (q & 7) ^ ((rl >> 1) & 7);             // logical chunk: entries 8 c .. 8 c + 7
        uint4 o = make_uint4(0u, 0u, 0u, 0u);     // rows of weight zero (padding too) are exact zeros
        if (w != 0.f) {
          o.x = pack_bf16(w * dz[i][0], w * dz[i][1]); o.y = pack_bf16(w * dz[i][2], w * dz[i][3]);
          o.z = pack_bf16(w * dz[i][4], w * dz[i][5]); o.w = pack_bf16(w * dz[i][6], w * dz[i][7]);
        }
        *(uint4*)&tile[rl][c * 8] = o;
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int u = i * 256 + threadIdx.x;
        const int j = u >> 9, vl = (u >> 3) & 63, pos = u & 7;
        const int imgrow = row0 + vl;
        const int c = pos ^ ((imgrow >> 1) & 7);             // slab rows 64 j + 8 c .. + 7
        const int rl = j * kBK + c * 8;
        uint4 o;
        o.x = tile[rl + 0][vl] | ((uint32_t)tile[rl + 1][vl] << 16);
        o.y = tile[rl + 2][vl] | ((uint32_t)tile[rl + 3][vl] << 16);
        o.z = tile[rl + 4][vl] | ((uint32_t)tile[rl + 5][vl] << 16);
        o.w = tile[rl + 6][vl] | ((uint32_t)tile[rl + 7][vl] << 16);
        dst[(((int64_t)vt * a.nkr + 4 * rt + j) * kGradTile + imgrow) * 8 + pos] = o;
      }
    }
  }
}

// Tile images of the transpose of the student hidden states of one slab, the B operand of
// the head-weight GEMMs: image row = hidden column (tiles of 256), k = slab row; entry =
// h_s[row_idx[r0 + r]][h] (zero beyond H).  One workgroup per (k-step of 64 rows, hidden tile).

__global__ __launch_bounds__(256) void hst_image_kernel(HstImageArgs a) {
  __shared__ uint16_t tile[kBK][kGradTile + 2];
  const int kr = blockIdx.x, ht = blockIdx.y, tid = threadIdx.x;
  for (int i = 0; i < kBK; ++i) {
    const int64_t r = a.row0 + (int64_t)kr * kBK + i;
    const int h = ht * kGradTile + tid;
    // an excluded row carries weight 0 in the other operand; its own entries (possibly inf or
    // NaN) must not meet that 0 in the product
    tile[i][tid] = (h < a.H && a.alive[r] != 0.f) ? a.h_s[(int64_t)a.row_idx[r] * a.H + h] : (uint16_t)0;
  }
  __syncthreads();
  uint16_t* blk = a.img + ((int64_t)ht * a.nkr + kr) * kImgElems;
  for (int q = tid; q < kGradTile * 8; q += 256) {
    const int r = q >> 3, pos = q & 7, c = pos ^ ((r >> 1) & 7);
    uint4 o;
    o.x = tile[c * 8 + 0][r] | ((uint32_t)tile[c * 8 + 1][r] << 16);
    o.y = tile[c * 8 + 2][r] | ((uint32_t)tile[c * 8 + 3][r] << 16);
    o.z = tile[c * 8 + 4][r] | ((uint32_t)tile[c * 8 + 5][r] << 16);
    o.w = tile[c * 8 + 6][r] | ((uint32_t)tile[c * 8 + 7][r] << 16);
    *(uint4*)(blk + q * 8) = o;
  }
}

// ---------------------------------------------------------------------------------------
// Pass 3: g[r][h] = sum_v dz[r][v] W_s[v][h].  256 x 256 output tile, 2 x 2 waves of
// 128 x 128.  A = slab rows (i = row), B = rows of W_s^T (j = hidden column, contiguous in
// g).  The k-steps (one 32 KiB block of each operand) go through five block buffers in the
// LDS, three for B and two for A, by direct global->LDS loads.  Per k-step a wave issues
// its 16 wave-loads of the k-step after next in the shadow of MFMAs (see grad_kstep), so
// that they have a k-step or more (upwards of 2000 matrix-pipe cycles) to land.  The one
// barrier per k-step sits before the last of the four k16 sub-steps: by then every fragment
// of the current blocks is in registers, so the last sub-step's MFMAs cover the LDS reads of
// the next blocks' first fragments and the matrix pipe never waits for LDS after a barrier.
// ---------------------------------------------------------------------------------------

// Five block buffers fill the 160 KiB of LDS: a ring of three for the B operand and a ring
// of two for the A operand.
constexpr int kGradRing3 = 3;
constexpr int kGradRing2Off = kGradRing3 * kImgBytes;         // the ring of two follows
constexpr int kGradLds = (kGradRing3 + 2) * kImgBytes;        // 160 KiB

// LOADS: in k-step s the B block of k-step s + 2 is loaded in sub-steps 1 and 2, four
// wave-loads behind the last MFMAs of each (`early`: into the third buffer of its ring, which
// no wave reads any more once it has passed the previous step's barrier; all eight in one
// sub-step, whichever, is 1 % slower) and the A block of k-step s + 2 in sub-step 3 (`late`: after this step's
// barrier, into the buffer of the ring of two that this step has just finished reading).
// The early operand has a lead of a k-step and a quarter to a half, the late one of one k-step.  Which
// operand gets which was measured: in `dz W_s` every XCD streams all of W_s^T (B) once per
// round of tiles while a slab block (A) is fetched by one XCD only, and the deeper lead on
// B is worth 2 % (on A 4 % against no third buffer at all).  Loads return in order: the wait
// before the barrier leaves the youngest eight, this step's early loads, in flight.
// Ring state (wave-uniform, LDS addresses that include the wave's KiB, which the loads want and
// the fragment offsets swA/swB take out again): r_a, r_b = the A and B buffers this k-step
// reads, on return those of the next k-step.  (pa, pb) = the blocks loaded by the previous
// k-step, on return those loaded by this one.  voffd[d] = 16 lane + 1024 wave + 4096 d.  The
// ring and address arithmetic sits in the shadows of the first MFMAs (see ring_next).
template <bool LOADS, bool LAST>
__device__ __forceinline__ void grad_kstep(f32x16 (&acc)[4][4], bf16x8 (&fa)[2][4], bf16x8 (&fb)[2][4],
                                           uint32_t& r_a, uint32_t& r_b, uint32_t a_begin, uint32_t a_end,
                                           uint32_t b_begin, uint32_t b_end, const uint32_t (&swA)[4],
                                           const uint32_t (&swB)[4], const uint32_t (&voffd)[8],
                                           uint32_t& pa_lo, uint32_t& pa_hi, uint32_t& pb_lo, uint32_t& pb_hi) {
  uint32_t r_a_nx = 0, r_b_nx = 0, r_b_wr = 0;
  uint32_t xa = 0, xb = 0;      // the lane's LDS addresses of its first A and B fragment of a sub-step
#define ADWIN_FENCE __builtin_amdgcn_sched_barrier(0);
#define ADWIN_MM(KK, I, J)                                                                    \
  acc[I][J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[(KK) & 1][I], fb[(KK) & 1][J],       \
                                                      acc[I][J], 0, 0, 0);                    \
  ADWIN_FENCE
  // side operation M (0..15) in the shadow of MFMA M of sub-step KK: fragment reads of the
  // next sub-step (from this step's buffers, in sub-step 3 from the next step's), the ring and
  // address arithmetic (sub-step 0), then (sub-steps 1, 2 and 3) the wave-loads of the k-step
  // after next: 4 KiB groups d = 0..7 of the early block, then of the late block
#define ADWIN_SIDE(KK, M)                                                                           \
  if constexpr ((M) < 8 && ((KK) < 3 || !LAST)) {                                                   \
    if constexpr ((M) == 0) {                                                                       \
      xa = ((KK) < 3 ? r_a : r_a_nx) + swA[((KK) + 1) & 3];                                         \
      xb = ((KK) < 3 ? r_b : r_b_nx) + swB[((KK) + 1) & 3];                                         \
      asm volatile("" : "+v"(xa), "+v"(xb));                                                        \
    }                                                                                               \
    if constexpr (((M) & 1) == 0)                                                                   \
      fa[((KK) + 1) & 1][((M) >> 1) & 3] = lds_frag(xa)[(((M) >> 1) & 3) * 32 * kRowBytes / 16]; \
    else                                                                                            \
      fb[((KK) + 1) & 1][((M) >> 1) & 3] = lds_frag(xb)[(((M) >> 1) & 3) * 32 * kRowBytes / 16]; \
    if constexpr ((KK) == 0 && (M) == 0 && !LAST) r_b_nx = ring_next<kImgBytes>(r_b, b_begin, b_end); \
    if constexpr ((KK) == 0 && (M) == 1 && !LAST) r_a_nx = ring_next<kImgBytes>(r_a, a_begin, a_end); \
    if constexpr ((KK) == 0 && (M) == 2 && LOADS) r_b_wr = ring_next<kImgBytes>(r_b_nx, b_begin, b_end); \
    if constexpr ((KK) == 0 && (M) == 3 && LOADS) addr_advance<kImgBytes>(pb_lo, pb_hi);            \
    if constexpr ((KK) == 0 && (M) == 4 && LOADS) addr_advance<kImgBytes>(pa_lo, pa_hi);            \
    ADWIN_FENCE                                                                                     \
  } else if constexpr (((KK) == 1 || (KK) == 2) && (M) >= 12 && LOADS) {                            \
    dma16_at<(((KK) - 1) * 4 + (M) - 12) * 4096>(r_b_wr, voffd[(((KK) - 1) * 4 + (M) - 12) & 7], addr_of(pb_lo, pb_hi)); \
    ADWIN_FENCE                                                                                     \
  } else if constexpr ((KK) == 3 && (M) >= 8 && LOADS) {                                            \
    dma16_at<((M) - 8) * 4096>(r_a, voffd[((M) - 8) & 7], addr_of(pa_lo, pa_hi));                         \
    ADWIN_FENCE                                                                                     \
  }
#define ADWIN_ROW(KK, I, M0)                                                    \
  ADWIN_MM(KK, I, 0) ADWIN_SIDE(KK, (M0) + 0) ADWIN_MM(KK, I, 1) ADWIN_SIDE(KK, (M0) + 1) \
  ADWIN_MM(KK, I, 2) ADWIN_SIDE(KK, (M0) + 2) ADWIN_MM(KK, I, 3) ADWIN_SIDE(KK, (M0) + 3)
#define ADWIN_SUB(KK) ADWIN_ROW(KK, 0, 0) ADWIN_ROW(KK, 1, 4) ADWIN_ROW(KK, 2, 8) ADWIN_ROW(KK, 3, 12)
  ADWIN_FENCE
  ADWIN_SUB(0)
  ADWIN_SUB(1)
  ADWIN_SUB(2)
  // every fragment of this stage is in registers; the next stage's loads must have landed
  // before its first fragments are read in the shadow of the last sub-step
  if constexpr (!LAST) {
    if constexpr (LOADS) asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __syncthreads();
  }
  ADWIN_FENCE
  ADWIN_SUB(3)
  if constexpr (!LAST) { r_a = r_a_nx; r_b = r_b_nx; }
#undef ADWIN_SUB
#undef ADWIN_ROW
#undef ADWIN_SIDE
#undef ADWIN_MM
#undef ADWIN_FENCE
}

// The eight wave-loads of one 32 KiB block into the buffer at lds_wave (its address + 1024 wave).
template <int... D>
__device__ __forceinline__ void dma_block(uint32_t lds_wave, const uint32_t (&voffd)[8], const char* blk,
                                          std::integer_sequence<int, D...>) {
  (dma16_at<D * 4096>(lds_wave, voffd[D], blk), ...);
}

__global__ __launch_bounds__(256) void grad_gemm_kernel(GradArgs a) {
  extern __shared__ __align__(16) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  int vid = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int tiles = a.row_tiles * a.h_tiles;
  const int split = vid / tiles;
  vid -= split * tiles;
  const int rt = vid / a.h_tiles, ht = vid % a.h_tiles;
  const int k_begin = (int)((int64_t)a.nk_total * split / a.ksplit);
  const int k_end = (int)((int64_t)a.nk_total * (split + 1) / a.ksplit);
  const int nk = k_end - k_begin;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;

  // wave-load d of a block covers its bytes [4096 d + 1024 wave, + 1024): lane l moves the
  // 16 bytes at offset 16 l of that KiB to the same place of the LDS stage
  uint32_t voffd[8];
#pragma unroll
  for (int d = 0; d < 8; ++d) {
    voffd[d] = (uint32_t)lane * 16u + (uint32_t)wave * 1024u + (uint32_t)d * 4096u;
    asm volatile("" : "+v"(voffd[d]));   // kept in registers, not recomputed at every load
  }
  const char* sA = (const char*)a.slab + ((int64_t)rt * a.nk_total + k_begin) * kImgBytes;
  const char* sB = (const char*)a.WsT + ((int64_t)ht * a.nk_total + k_begin) * kImgBytes;
  const uint32_t ldsw = lds0 + (uint32_t)wave * 1024u;
  // the ring of three (offset 0) holds the W_s^T blocks, the ring of two the slab blocks
  const uint32_t b_begin = ldsw, b_end = ldsw + kGradRing3 * kImgBytes;
  const uint32_t a_begin = ldsw + kGradRing2Off, a_end = a_begin + 2 * kImgBytes;
  const std::make_integer_sequence<int, 8> all8{};

  f32x16 acc[4][4];
#pragma unroll
  for (int fm = 0; fm < 4; ++fm)
#pragma unroll
    for (int fn = 0; fn < 4; ++fn)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[fm][fn][e] = 0.f;

  if (nk > 0) {
    // first the blocks of k-step 0, then its first fragments
    dma_block(b_begin, voffd, sB, all8);
    dma_block(a_begin, voffd, sA, all8);
    wait_vm<0>();
    __syncthreads();
    bf16x8 fa[2][4], fb[2][4];
    uint32_t swA[4], swB[4];
    {
      const int key = (lane >> 1) & 7, half = lane >> 5;
      const uint32_t rowoff = (uint32_t)(lane & 31) * kRowBytes - (uint32_t)wave * 1024u;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const uint32_t x = rowoff + (uint32_t)(((kk * 2 + half) ^ key) << 4);
        swA[kk] = x + (uint32_t)(wm * 128 * kRowBytes);
        swB[kk] = x + (uint32_t)(wn * 128 * kRowBytes);
      }
    }
    uint32_t r_a = a_begin, r_b = b_begin;     // k-step s reads B buffer s % 3 and A buffer s % 2
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      fa[0][i] = lds_frag(r_a + swA[0])[i * 32 * kRowBytes / 16];
      fb[0][i] = lds_frag(r_b + swB[0])[i * 32 * kRowBytes / 16];
    }
    // blocks of k-step 1 (k-step s of the loop loads those of k-step s + 2)
    uint64_t pa = (uint64_t)sA, pb = (uint64_t)sB;
    if (nk > 1) {
      pa += kImgBytes; pb += kImgBytes;
      dma_block(b_begin + kImgBytes, voffd, (const char*)pb, all8);
      dma_block(a_begin + kImgBytes, voffd, (const char*)pa, all8);
    }
    uint32_t pa_lo = (uint32_t)pa, pa_hi = (uint32_t)(pa >> 32), pb_lo = (uint32_t)pb, pb_hi = (uint32_t)(pb >> 32);
    int s = 0;
    for (; s + 2 < nk; ++s)
      grad_kstep<true, false>(acc, fa, fb, r_a, r_b, a_begin, a_end, b_begin, b_end, swA, swB, voffd,
                              pa_lo, pa_hi, pb_lo, pb_hi);
    if (s + 1 < nk)
      grad_kstep<false, false>(acc, fa, fb, r_a, r_b, a_begin, a_end, b_begin, b_end, swA, swB, voffd,
                               pa_lo, pa_hi, pb_lo, pb_hi);
    grad_kstep<false, true>(acc, fa, fb, r_a, r_b, a_begin, a_end, b_begin, b_end, swA, swB, voffd,
                            pa_lo, pa_hi, pb_lo, pb_hi);
  }
  float* g = a.g + (int64_t)split * a.g_rows * a.H;
  const int64_t out_row0 = rt < a.half_tiles ? a.slab_row0 + (int64_t)rt * kGradTile
                                             : a.half_off + a.slab_row0 + (int64_t)(rt - a.half_tiles) * kGradTile;
#pragma unroll
  for (int fm = 0; fm < 4; ++fm)
#pragma unroll
    for (int fn = 0; fn < 4; ++fn) {
      const int h = ht * kGradTile + wn * 128 + fn * 32 + (lane & 31);
      if (h < a.H) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int64_t r = out_row0 + wm * 128 + fm * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
          if (r < a.out_rows) {
            float* o = g + r * a.H + h;
            // accumulate: every element is added to by exactly one lane of this launch and
            // launches are ordered on the stream, so the hardware add keeps the sum
            // deterministic while sparing the lane the round trip of a load
            if (a.accumulate) unsafeAtomicAdd(o, acc[fm][fn][e]);
            else *o = acc[fm][fn][e];
          }
        }
      }
    }
}

// ---------------------------------------------------------------------------------------
// Finalize: one wave per packed row.  Sums the k-split partials, writes the row norm,
// scales by grad_scale*alpha and scatters to dh_prefix / dh_full (zero outside windows).
// ---------------------------------------------------------------------------------------

__device__ __forceinline__ void store_dh(void* base, int bf16, int64_t t, int H, int h, float4 v) {
  if (!base) return;
  if (bf16) {
    uint2 o;
    o.x = pack_bf16(v.x, v.y);
    o.y = pack_bf16(v.z, v.w);
    *(uint2*)((uint16_t*)base + t * H + h) = o;
  } else {
    *(float4*)((float*)base + t * H + h) = v;
  }
}

__global__ __launch_bounds__(256) void finalize_kernel(FinalizeArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= a.T) return;
  const int i = last_le<int64_t>(a.pl.offsets, a.B + 1, t);
  const int64_t j = t - a.pl.offsets[i];
  const bool admitted = j < a.pl.n[i];
  const bool computed = a.probe || admitted;
  const float4 zero = {0.f, 0.f, 0.f, 0.f};
  if (!computed) {
    for (int h = lane * 4; h < a.H; h += 256) store_dh(a.dh_prefix, a.dh_bf16, t, a.H, h, zero);
    return;
  }
  const int64_t r = a.pl.comp_off[i] + j;
  if (a.inv_z[r] == 0.f) {
    // excluded row (no finite statistics): zeros in both gradients, in g (the pooled sums
    // read it) and in the row norm
    for (int h = lane * 4; h < a.H; h += 256) {
      *(float4*)(a.g + r * a.H + h) = zero;
      store_dh(a.dh_prefix, a.dh_bf16, t, a.H, h, zero);
      if (a.probe) store_dh(a.dh_full, a.dh_bf16, t, a.H, h, zero);
    }
    if (lane == 0) a.rownorm[r] = 0.f;
    return;
  }
  const float sp = admitted ? a.grad_scale * a.pl.alpha_p[i] : 0.f;
  const float sf = a.grad_scale * a.pl.alpha_f[i];
  float nrm = 0.f;
  if (a.cr) {
    const float c = a.cr[r], iz = a.inv_z[r];
    const int y = a.ids[t];
    const bool ok = y >= 0 && y < a.V;            // c is 0 otherwise
    const uint2* wy = (const uint2*)(a.W_s + (int64_t)(ok ? y : 0) * a.H);
    for (int h = lane * 4; h < a.H; h += 256) {
      float4 g2 = *(const float4*)(a.g + (a.n_pad + r) * a.H + h);
      for (int s = 1; s < a.ksplit; ++s) {
        const float4 q = *(const float4*)(a.g + ((int64_t)s * a.g_rows + a.n_pad + r) * a.H + h);
        g2.x += q.x; g2.y += q.y; g2.z += q.z; g2.w += q.w;
      }
      const uint2 w = wy[h >> 2];
      float4 g;
      g.x = c * (bf16_lo(w.x) - g2.x * iz); g.y = c * (bf16_hi(w.x) - g2.y * iz);
      g.z = c * (bf16_lo(w.y) - g2.z * iz); g.w = c * (bf16_hi(w.y) - g2.w * iz);
      *(float4*)(a.g + r * a.H + h) = g;
      nrm = fmaf(g.x, g.x, fmaf(g.y, g.y, fmaf(g.z, g.z, fmaf(g.w, g.w, nrm))));
      const float4 p = {g.x * sp, g.y * sp, g.z * sp, g.w * sp};
      store_dh(a.dh_prefix, a.dh_bf16, t, a.H, h, p);
      if (a.probe) {
        const float4 f = {g.x * sf, g.y * sf, g.z * sf, g.w * sf};
        store_dh(a.dh_full, a.dh_bf16, t, a.H, h, f);
      }
    }
    nrm = wave_sum(nrm);
    if (lane == 0) a.rownorm[r] = nrm;
    return;
  }
  // Heavy entries of the row (those the bf16 operand holds as zeros): lane k ends up with the
  // k-th smallest listed vocabulary index hv and that entry's logit gradient hd, taken in fp32
  // from fresh dot products.  The list is filled in no particular order; adding the entries in
  // index order keeps the result the same from call to call.
  int nh = a.heavy.cnt ? a.heavy.cnt[r] : 0;
  nh = nh < kHeavySlots ? nh : kHeavySlots;
  int hv = 0;
  float hd = 0.f;
  if (nh > 0) {
    const int mine = lane < nh ? a.heavy.v[r * kHeavySlots + lane] : 0x7fffffff;
    int rank = 0;                                  // indices of one row are distinct
    for (int k = 0; k < nh; ++k) rank += (__shfl(mine, k, 64) < mine) ? 1 : 0;
    for (int k = 0; k < nh; ++k) {
      const int vk = __shfl(mine, k, 64), rk = __shfl(rank, k, 64);
      if (rk == lane) hv = vk;
    }
    const float lse = a.lse_s[r], mu = a.mu[r];
    for (int k = 0; k < nh; ++k) {
      const int v = __shfl(hv, k, 64);
      const float zs = dot_bf16_row(a.h_s + t * a.H, a.W_s + (int64_t)v * a.H, a.H, lane);
      const float zt = dot_bf16_row(a.h_t + t * a.H_t, a.W_t + (int64_t)v * a.H_t, a.H_t, lane);
      if (lane == k) hd = __expf(zs - lse) * ((zs - zt) - mu);
    }
  }
  for (int h0 = 0; h0 < a.H; h0 += 256) {          // every lane takes part in the shuffles
    const int h = h0 + lane * 4;
    const bool act = h < a.H;
    float4 g = zero;
    if (act) {
      g = *(const float4*)(a.g + r * a.H + h);
      for (int s = 1; s < a.ksplit; ++s) {
        const float4 q = *(const float4*)(a.g + ((int64_t)s * a.g_rows + r) * a.H + h);
        g.x += q.x; g.y += q.y; g.z += q.z; g.w += q.w;
      }
    }
    for (int k = 0; k < nh; ++k) {
      const int v = __shfl(hv, k, 64);
      const float dzv = __shfl(hd, k, 64);
      if (act) {
        const uint2 w = *(const uint2*)(a.W_s + (int64_t)v * a.H + h);
        g.x = fmaf(dzv, bf16_lo(w.x), g.x); g.y = fmaf(dzv, bf16_hi(w.x), g.y);
        g.z = fmaf(dzv, bf16_lo(w.y), g.z); g.w = fmaf(dzv, bf16_hi(w.y), g.w);
      }
    }
    if (act) {
      if (a.ksplit > 1 || nh > 0) *(float4*)(a.g + r * a.H + h) = g;
      nrm = fmaf(g.x, g.x, fmaf(g.y, g.y, fmaf(g.z, g.z, fmaf(g.w, g.w, nrm))));
      const float4 p = {g.x * sp, g.y * sp, g.z * sp, g.w * sp};
      store_dh(a.dh_prefix, a.dh_bf16, t, a.H, h, p);
      if (a.probe) {
        const float4 f = {g.x * sf, g.y * sf, g.z * sf, g.w * sf};
        store_dh(a.dh_full, a.dh_bf16, t, a.H, h, f);
      }
    }
  }
  nrm = wave_sum(nrm);
  if (lane == 0) a.rownorm[r] = nrm;
}

// ---------------------------------------------------------------------------------------
// Pooled gradients: column sums of g over the window and over the rollout, two levels.
// ---------------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void pool_partial_kernel(PoolArgs a) {
  const int ch = blockIdx.x;
  const int h = blockIdx.y * 256 + threadIdx.x;
  const int i = last_le<int32_t>(a.pl.chunk_off, a.B + 1, ch);
  const int64_t len = a.pl.offsets[i + 1] - a.pl.offsets[i];
  const int64_t ni = a.pl.n[i];
  const int64_t hi = a.probe ? len : ni;
  const int64_t j0 = (int64_t)(ch - a.pl.chunk_off[i]) * kChunkRows;
  const int64_t j1 = j0 + kChunkRows < hi ? j0 + kChunkRows : hi;
  if (h >= a.H) return;
  const float* g = a.g + (a.pl.comp_off[i] + j0) * a.H + h;
  float sp = 0.f, sf = 0.f;
  for (int64_t j = j0; j < j1; ++j, g += a.H) {
    const float v = *g;
    sf += v;
    if (j < ni) sp += v;
  }
  a.pp[(int64_t)ch * a.H + h] = sp;
  a.pf[(int64_t)ch * a.H + h] = sf;
}

__global__ __launch_bounds__(256) void pool_final_kernel(PoolArgs a) {
  const int i = blockIdx.x;
  const int h = blockIdx.y * 256 + threadIdx.x;
  if (h >= a.H) return;
  float sp = 0.f, sf = 0.f;
  for (int ch = a.pl.chunk_off[i]; ch < a.pl.chunk_off[i + 1]; ++ch) {
    sp += a.pp[(int64_t)ch * a.H + h];
    sf += a.pf[(int64_t)ch * a.H + h];
  }
  a.up[(int64_t)i * a.H + h] = sp;
  a.uf[(int64_t)i * a.H + h] = sf;
}

// ---------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------
hipError_t grad_kernels_opt_in() {
  return hipFuncSetAttribute((const void*)grad_gemm_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                             kGradLds);
}

hipError_t launch_wst_image(const void* W_s, void* img, int V, int H, int nk, int h_tiles, hipStream_t st) {
  wst_image_kernel<<<dim3((unsigned)nk, (unsigned)h_tiles), 256, 0, st>>>((const uint16_t*)W_s, (uint16_t*)img,
                                                                          V, H, nk);
  return hipGetLastError();
}

hipError_t launch_hst_image(const HstImageArgs& a, int h_tiles, hipStream_t st) {
  hst_image_kernel<<<dim3((unsigned)a.nkr, (unsigned)h_tiles), 256, 0, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_combine(bool transposed, bool sampled, const CombineArgs& a, int row_tiles, hipStream_t st) {
  const dim3 grid((unsigned)a.nk, (unsigned)row_tiles);
  if (sampled) {
    if (!transposed) return hipErrorInvalidValue;   // the sampled estimator contracts E2 as stored
    combine_kernel<true, true><<<grid, 256, 0, st>>>(a);
  } else if (transposed) {
    combine_kernel<true><<<grid, 256, 0, st>>>(a);
  } else {
    combine_kernel<false><<<grid, 256, 0, st>>>(a);
  }
  return hipGetLastError();
}

hipError_t launch_grad_gemm(const GradArgs& a, hipStream_t st) {
  grad_gemm_kernel<<<(unsigned)(a.row_tiles * a.h_tiles * a.ksplit), 256, kGradLds, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_finalize(const FinalizeArgs& a, hipStream_t st) {
  finalize_kernel<<<(unsigned)((a.T + 3) / 4), 256, 0, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_pool_partial(const PoolArgs& a, int n_chunks, hipStream_t st) {
  pool_partial_kernel<<<dim3((unsigned)n_chunks, (unsigned)((a.H + 255) / 256)), 256, 0, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_pool_final(const PoolArgs& a, hipStream_t st) {
  pool_final_kernel<<<dim3((unsigned)a.B, (unsigned)((a.H + 255) / 256)), 256, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace adwin
