// Plan expansion, fills and the deterministic segmented reductions over ragged
// windows: per-window losses (Sec. 4.1) and prefix-vs-full alignment (Sec. 4.2).
// No floating-point atomics: every sum has a fixed order.
#include <cmath>
#include <cstring>

#include "device_utils.h"
#include "plan_device.h"

namespace adwin {

DevicePlan device_plan_at(unsigned char* ws_plan, int32_t B, int32_t* row_idx, int32_t* row_seq) {
  PlanBlobLayout L(B);
  DevicePlan d;
  d.offsets = (const int64_t*)(ws_plan + L.o_offsets);
  d.comp_off = (const int64_t*)(ws_plan + L.o_comp_off);
  d.n = (const int32_t*)(ws_plan + L.o_n);
  d.chunk_off = (const int32_t*)(ws_plan + L.o_chunk_off);
  d.alpha_p = (const float*)(ws_plan + L.o_alpha_p);
  d.alpha_f = (const float*)(ws_plan + L.o_alpha_f);
  d.row_idx = row_idx;
  d.row_seq = row_seq;
  return d;
}

// ---------------------------------------------------------------------------------------
// small kernels
// ---------------------------------------------------------------------------------------
__global__ void build_rows_kernel(DevicePlan pl, int B, int64_t n_rows, int64_t n_pad) {
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_pad) return;
  const int64_t rr = r < n_rows ? r : n_rows - 1;   // padding repeats the last computed row
  const int i = last_le<int64_t>(pl.comp_off, B + 1, rr);
  pl.row_idx[r] = (int32_t)(pl.offsets[i] + (rr - pl.comp_off[i]));
  pl.row_seq[r] = i;
}

__global__ void fill_f32_kernel(float* p, int64_t n, float v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
__global__ void fill_u32_kernel(uint32_t* p, int64_t n, uint32_t v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// Fixed-order block sum of up to 4 doubles per thread (256 threads).
template <int K>
__device__ __forceinline__ void block_sum256(double (&v)[K], double* sh /* [K][4] */) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int k = 0; k < K; ++k) {
    v[k] = wave_sum(v[k]);
    if (lane == 0) sh[k * 4 + w] = v[k];
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < K; ++k) v[k] = (sh[k * 4 + 0] + sh[k * 4 + 1]) + (sh[k * 4 + 2] + sh[k * 4 + 3]);
  __syncthreads();
}

// One workgroup per rollout: sums of KL_t and ||g_t||^2 over the window and the rollout.
__global__ __launch_bounds__(256) void segment_sums_kernel(DevicePlan pl, int probe,
                                                           const float* __restrict__ klr,
                                                           const float* __restrict__ rownorm,
                                                           double* __restrict__ seg,
                                                           float* loss_prefix, float* loss_full) {
  __shared__ double sh[16];
  const int i = blockIdx.x;
  const int64_t len = pl.offsets[i + 1] - pl.offsets[i];
  const int64_t ni = pl.n[i];
  const int64_t hi = probe ? len : ni;
  const int64_t r0 = pl.comp_off[i];
  double v[4] = {0.0, 0.0, 0.0, 0.0};   // kl prefix, kl full, norm prefix, norm full
  for (int64_t j = threadIdx.x; j < hi; j += 256) {
    const double k = klr[r0 + j];
    const double s = rownorm ? (double)rownorm[r0 + j] : 0.0;
    v[1] += k;
    v[3] += s;
    if (j < ni) { v[0] += k; v[2] += s; }
  }
  block_sum256<4>(v, sh);
  if (threadIdx.x == 0) {
    seg[i * 4 + 0] = v[0];
    seg[i * 4 + 1] = v[1];
    seg[i * 4 + 2] = v[2];
    seg[i * 4 + 3] = v[3];
    if (loss_prefix) loss_prefix[i] = ni > 0 ? (float)(v[0] / (double)ni) : 0.f;
    if (loss_full) loss_full[i] = (probe && len > 0) ? (float)(v[1] / (double)len) : 0.f;
  }
}

// One workgroup per rollout: cosines from the pooled sums and the norm sums.
__global__ __launch_bounds__(256) void rollout_alignment_kernel(BatchArgs a) {
  __shared__ double sh[16];
  const int i = blockIdx.x;
  double v[3] = {0.0, 0.0, 0.0};
  if (a.probe && !a.zero_grad) {
    const float* up = a.up + (size_t)i * a.H;
    const float* uf = a.uf + (size_t)i * a.H;
    for (int h = threadIdx.x; h < a.H; h += 256) {
      const double p = up[h], f = uf[h];
      v[0] += p * f;
      v[1] += p * p;
      v[2] += f * f;
    }
  }
  block_sum256<3>(v, sh);
  if (threadIdx.x == 0) {
    double rp = 0.0, rf = 0.0, okp = 0.0, okf = 0.0;
    if (a.probe && !a.zero_grad) {
      if (v[1] > 0.0 && v[2] > 0.0) { rp = v[0] / (sqrt(v[1]) * sqrt(v[2])); okp = 1.0; }
      const double Sp = a.seg[i * 4 + 2], Sf = a.seg[i * 4 + 3];
      if (Sp > 0.0 && Sf > 0.0) { rf = sqrt(Sp / Sf); okf = 1.0; }
    }
    a.racc[i * 4 + 0] = rp;
    a.racc[i * 4 + 1] = okp;
    a.racc[i * 4 + 2] = rf;
    a.racc[i * 4 + 3] = okf;
    if (a.rho_pooled) a.rho_pooled[i] = (float)rp;
    if (a.rho_field) a.rho_field[i] = (float)rf;
  }
}

// Single workgroup: batch objectives, micro (after aggregation) and macro (mean of
// per-rollout) alignment, integer outputs.
__global__ __launch_bounds__(256) void batch_kernel(BatchArgs a) {
  __shared__ double sh[16];
  const int B = a.B;
  // batch objectives and field sums
  double w[4] = {0.0, 0.0, 0.0, 0.0};   // L^p, L^f, macro pooled sum, macro pooled count
  double f[4] = {0.0, 0.0, 0.0, 0.0};   // field: dot, |p|^2, |f|^2, unused
  double mf[2] = {0.0, 0.0};            // macro field sum, count
  for (int i = threadIdx.x; i < B; i += 256) {
    const double ap = a.pl.alpha_p[i], af = a.pl.alpha_f[i];
    w[0] += ap * a.seg[i * 4 + 0];
    if (a.probe) {
      w[1] += af * a.seg[i * 4 + 1];
      w[2] += a.racc[i * 4 + 0] * a.racc[i * 4 + 1];
      w[3] += a.racc[i * 4 + 1];
      mf[0] += a.racc[i * 4 + 2] * a.racc[i * 4 + 3];
      mf[1] += a.racc[i * 4 + 3];
      const double Sp = a.seg[i * 4 + 2], Sf = a.seg[i * 4 + 3];
      f[0] += ap * af * Sp;
      f[1] += ap * ap * Sp;
      f[2] += af * af * Sf;
    }
  }
  block_sum256<4>(w, sh);
  block_sum256<4>(f, sh);
  block_sum256<2>(mf, sh);
  // micro pooled: aggregate the weighted pooled gradients over the batch, then one cosine
  double m[3] = {0.0, 0.0, 0.0};
  if (a.probe && !a.zero_grad) {
    for (int h = threadIdx.x; h < a.H; h += 256) {
      double sp = 0.0, sf = 0.0;
      for (int i = 0; i < B; ++i) {
        sp += (double)a.pl.alpha_p[i] * (double)a.up[(size_t)i * a.H + h];
        sf += (double)a.pl.alpha_f[i] * (double)a.uf[(size_t)i * a.H + h];
      }
      m[0] += sp * sf;
      m[1] += sp * sp;
      m[2] += sf * sf;
    }
  }
  block_sum256<3>(m, sh);
  if (a.n_out)
    for (int i = threadIdx.x; i < B; i += 256) a.n_out[i] = a.pl.n[i];
  if (threadIdx.x == 0) {
    if (a.n_adm_out) *a.n_adm_out = a.n_adm;
    if (a.batch) {
      float o[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      o[0] = (float)w[0];
      if (a.probe) {
        o[1] = (float)w[1];
        if (!a.zero_grad) {
          if (m[1] > 0.0 && m[2] > 0.0) o[2] = (float)(m[0] / (sqrt(m[1]) * sqrt(m[2])));
          if (f[1] > 0.0 && f[2] > 0.0) o[3] = (float)(f[0] / (sqrt(f[1]) * sqrt(f[2])));
          if (w[3] > 0.0) o[4] = (float)(w[2] / w[3]);
          if (mf[1] > 0.0) o[5] = (float)(mf[0] / mf[1]);
        }
      }
      for (int k = 0; k < 8; ++k) a.batch[k] = o[k];
    }
  }
}

// ---------------------------------------------------------------------------------------
// Candidate-window audit (Sec. 4.2).  For candidate k every rollout uses the shared window
// L_k: n = min(L_k, len_i).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ double cand_alpha_p(const CandArgs& a, int k, int64_t n) {
  if (n <= 0) return 0.0;
  if (a.reduction == ADWIN_RED_SEQ_MEAN) return 1.0 / ((double)a.B * (double)n);
  if (a.reduction == ADWIN_RED_SUM) return 1.0;
  return a.inv_nadm[k];
}

// Pooled prefix sum u_i(L_k): whole chunks from the chunk sums, the ragged rest row by row.
__global__ __launch_bounds__(256) void cand_pool_kernel(CandArgs a) {
  const int k = blockIdx.x / a.B, i = blockIdx.x % a.B;
  const int h = blockIdx.y * 256 + threadIdx.x;
  if (h >= a.H) return;
  const int64_t len = a.pl.offsets[i + 1] - a.pl.offsets[i];
  const int64_t n = a.L[k] < len ? (int64_t)a.L[k] : len;
  const int64_t full = n / kChunkRows;
  float s = 0.f;
  const float* pf = a.pf + (int64_t)a.pl.chunk_off[i] * a.H + h;
  for (int64_t c = 0; c < full; ++c) s += pf[c * a.H];
  const float* g = a.g + (a.pl.comp_off[i] + full * kChunkRows) * a.H + h;
  for (int64_t j = full * kChunkRows; j < n; ++j, g += a.H) s += *g;
  a.uc[((int64_t)k * a.B + i) * a.H + h] = s;
}

// One workgroup per (candidate, rollout): cosines of the pooled and of the field gradients.
__global__ __launch_bounds__(256) void cand_align_kernel(CandArgs a) {
  __shared__ double sh[16];
  const int k = blockIdx.x / a.B, i = blockIdx.x % a.B;
  const int64_t len = a.pl.offsets[i + 1] - a.pl.offsets[i];
  const int64_t n = a.L[k] < len ? (int64_t)a.L[k] : len;
  double v[4] = {0.0, 0.0, 0.0, 0.0};   // <u_p,u_f>, |u_p|^2, |u_f|^2, S_i(n)
  if (!a.zero_grad) {
    const float* up = a.uc + ((int64_t)k * a.B + i) * a.H;
    const float* uf = a.uf + (int64_t)i * a.H;
    for (int h = threadIdx.x; h < a.H; h += 256) {
      const double p = up[h], f = uf[h];
      v[0] += p * f;
      v[1] += p * p;
      v[2] += f * f;
    }
    const float* rn = a.rownorm + a.pl.comp_off[i];
    for (int64_t j = threadIdx.x; j < n; j += 256) v[3] += (double)rn[j];
  }
  block_sum256<4>(v, sh);
  if (threadIdx.x == 0) {
    double rp = 0.0, rf = 0.0, okp = 0.0, okf = 0.0;
    if (!a.zero_grad) {
      if (v[1] > 0.0 && v[2] > 0.0) { rp = v[0] / (sqrt(v[1]) * sqrt(v[2])); okp = 1.0; }
      const double Sf = a.seg[i * 4 + 3];
      if (v[3] > 0.0 && Sf > 0.0) { rf = sqrt(v[3] / Sf); okf = 1.0; }
    }
    const int64_t o = (int64_t)k * a.B + i;
    a.cacc[o * 4 + 0] = rp;
    a.cacc[o * 4 + 1] = okp;
    a.cacc[o * 4 + 2] = rf;
    a.cacc[o * 4 + 3] = okf;
    a.cS[o] = v[3];
    if (a.rho_pooled) a.rho_pooled[o] = (float)rp;
    if (a.rho_field) a.rho_field[o] = (float)rf;
  }
}

// One workgroup per candidate: micro (after batch aggregation) and macro cosines.
__global__ __launch_bounds__(256) void cand_batch_kernel(CandArgs a) {
  __shared__ double sh[16];
  const int k = blockIdx.x, B = a.B;
  double w[4] = {0.0, 0.0, 0.0, 0.0};   // macro pooled sum, count, macro field sum, count
  double f[3] = {0.0, 0.0, 0.0};        // field: dot, |p|^2, |f|^2
  for (int i = threadIdx.x; i < B; i += 256) {
    const int64_t o = (int64_t)k * B + i;
    const int64_t len = a.pl.offsets[i + 1] - a.pl.offsets[i];
    const int64_t n = a.L[k] < len ? (int64_t)a.L[k] : len;
    const double ap = cand_alpha_p(a, k, n), af = a.pl.alpha_f[i];
    w[0] += a.cacc[o * 4 + 0] * a.cacc[o * 4 + 1];
    w[1] += a.cacc[o * 4 + 1];
    w[2] += a.cacc[o * 4 + 2] * a.cacc[o * 4 + 3];
    w[3] += a.cacc[o * 4 + 3];
    f[0] += ap * af * a.cS[o];
    f[1] += ap * ap * a.cS[o];
    f[2] += af * af * a.seg[i * 4 + 3];
  }
  block_sum256<4>(w, sh);
  block_sum256<3>(f, sh);
  double m[3] = {0.0, 0.0, 0.0};
  if (!a.zero_grad) {
    for (int h = threadIdx.x; h < a.H; h += 256) {
      double sp = 0.0, sf = 0.0;
      for (int i = 0; i < B; ++i) {
        const int64_t len = a.pl.offsets[i + 1] - a.pl.offsets[i];
        const int64_t n = a.L[k] < len ? (int64_t)a.L[k] : len;
        sp += cand_alpha_p(a, k, n) * (double)a.uc[((int64_t)k * B + i) * a.H + h];
        sf += (double)a.pl.alpha_f[i] * (double)a.uf[(int64_t)i * a.H + h];
      }
      m[0] += sp * sf;
      m[1] += sp * sp;
      m[2] += sf * sf;
    }
  }
  block_sum256<3>(m, sh);
  if (threadIdx.x == 0 && a.batch) {
    float o[4] = {0.f, 0.f, 0.f, 0.f};
    if (!a.zero_grad) {
      if (m[1] > 0.0 && m[2] > 0.0) o[0] = (float)(m[0] / (sqrt(m[1]) * sqrt(m[2])));
      if (f[1] > 0.0 && f[2] > 0.0) o[1] = (float)(f[0] / (sqrt(f[1]) * sqrt(f[2])));
      if (w[1] > 0.0) o[2] = (float)(w[0] / w[1]);
      if (w[3] > 0.0) o[3] = (float)(w[2] / w[3]);
    }
    for (int q = 0; q < 4; ++q) a.batch[k * 4 + q] = o[q];
  }
}


// ---------------------------------------------------------------------------------------
// Rollout-level summaries of the per-row outputs.  One workgroup per rollout; every thread
// takes positions tid, tid + 256, ... in ascending order with double accumulators, and the
// 256 partials are folded by a fixed tree, so the results do not depend on scheduling.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ double block_sum_256(double v, double* sh) {
  const int tid = threadIdx.x;
  sh[tid] = v;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) sh[tid] += sh[tid + s];
    __syncthreads();
  }
  const double r = sh[0];
  __syncthreads();
  return r;
}

__global__ __launch_bounds__(256) void summary_rollout_kernel(SummaryArgs a) {
  __shared__ double sh[256];
  __shared__ int sh_first[256];
  const int i = blockIdx.x, tid = threadIdx.x;
  const int64_t base = a.pl.offsets[i];
  const int64_t len = a.pl.offsets[i + 1] - base;
  const int64_t n = a.pl.n[i];
  const int64_t m = a.probe ? len : n;          // computed positions of this rollout
  double* acc = a.acc + (size_t)i * kSummarySlots;
  if (a.first_reject) {
    int64_t first = m;
    for (int64_t j = tid; j < m; j += 256)
      if (a.t_rank[base + j] > a.topk) { first = j; break; }
    sh_first[tid] = (int)first;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
      if (tid < s) sh_first[tid] = min(sh_first[tid], sh_first[tid + s]);
      __syncthreads();
    }
    if (tid == 0) a.first_reject[i] = sh_first[0];
    __syncthreads();
  }
  if (a.logp_mean) {
    double sp = 0.0, ss = 0.0;
    for (int64_t j = tid; j < m; j += 256) {
      const double v = (double)a.t_logp[base + j];
      if (j < n) sp += v; else ss += v;
    }
    sp = block_sum_256(sp, sh);
    ss = block_sum_256(ss, sh);
    if (tid == 0) {
      acc[ADWIN_MAX_CANDIDATES + 1] = sp;
      acc[ADWIN_MAX_CANDIDATES + 2] = ss;
      a.logp_mean[2 * i + 0] = n > 0 ? (float)(sp / (double)n) : 0.f;
      a.logp_mean[2 * i + 1] = m > n ? (float)(ss / (double)(m - n)) : 0.f;
    }
  }
  if (a.loss_share) {
    double part[ADWIN_MAX_CANDIDATES];
#pragma unroll
    for (int k = 0; k < ADWIN_MAX_CANDIDATES; ++k) part[k] = 0.0;
    double tot = 0.0;
    for (int64_t j = tid; j < m; j += 256) {
      const double v = (double)a.kl[base + j];
      tot += v;
#pragma unroll
      for (int k = 0; k < ADWIN_MAX_CANDIDATES; ++k)
        if (k < a.K && j < a.L[k]) part[k] += v;
    }
    tot = block_sum_256(tot, sh);
    if (tid == 0) acc[ADWIN_MAX_CANDIDATES] = tot;
#pragma unroll
    for (int k = 0; k < ADWIN_MAX_CANDIDATES; ++k) {
      if (k < a.K) {                              // uniform across the workgroup
        const double r = block_sum_256(part[k], sh);
        if (tid == 0) acc[k] = r;
      }
    }
  }
}

// Batch rows of the summaries: sums over rollouts in index order.
__global__ __launch_bounds__(64) void summary_batch_kernel(SummaryArgs a) {
  const int tid = threadIdx.x;
  if (a.loss_share && tid < a.K) {
    double part = 0.0, tot = 0.0;
    for (int i = 0; i < a.B; ++i) {
      part += a.acc[(size_t)i * kSummarySlots + tid];
      tot += a.acc[(size_t)i * kSummarySlots + ADWIN_MAX_CANDIDATES];
    }
    a.loss_share[tid] = tot != 0.0 ? (float)(part / tot) : 0.f;
  }
  if (a.logp_mean && tid >= 32 && tid < 34) {
    const int c = tid - 32;
    double sum = 0.0;
    int64_t cnt = 0;
    for (int i = 0; i < a.B; ++i) {
      const int64_t len = a.pl.offsets[i + 1] - a.pl.offsets[i];
      const int64_t n = a.pl.n[i], m = a.probe ? len : n;
      sum += a.acc[(size_t)i * kSummarySlots + ADWIN_MAX_CANDIDATES + 1 + c];
      cnt += c == 0 ? n : m - n;
    }
    a.logp_mean[2 * a.B + c] = cnt > 0 ? (float)(sum / (double)cnt) : 0.f;
  }
}

// ---------------------------------------------------------------------------------------
// Cosine of two long fp32 arrays (the two head-weight gradients).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void cosine_partial_kernel(const float* x, const float* y, int64_t n,
                                                             double* partials) {
  __shared__ double sh[256];
  const int64_t per = (n + kCosineBlocks - 1) / kCosineBlocks;
  const int64_t lo = (int64_t)blockIdx.x * per;
  const int64_t hi = lo + per < n ? lo + per : n;
  double xy = 0.0, xx = 0.0, yy = 0.0;
  for (int64_t q = lo + threadIdx.x; q < hi; q += 256) {
    const double a = (double)x[q], b = (double)y[q];
    xy += a * b; xx += a * a; yy += b * b;
  }
  xy = block_sum_256(xy, sh);
  xx = block_sum_256(xx, sh);
  yy = block_sum_256(yy, sh);
  if (threadIdx.x == 0) {
    partials[3 * blockIdx.x + 0] = xy;
    partials[3 * blockIdx.x + 1] = xx;
    partials[3 * blockIdx.x + 2] = yy;
  }
}

__global__ void cosine_final_kernel(const double* partials, float* out) {
  if (threadIdx.x != 0) return;
  double xy = 0.0, xx = 0.0, yy = 0.0;
  for (int b = 0; b < kCosineBlocks; ++b) {
    xy += partials[3 * b + 0]; xx += partials[3 * b + 1]; yy += partials[3 * b + 2];
  }
  *out = (xx > 0.0 && yy > 0.0) ? (float)(xy / (sqrt(xx) * sqrt(yy))) : 0.f;
}

// ---------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------
hipError_t launch_cosine(const float* x, const float* y, int64_t n, double* partials, float* out,
                         hipStream_t st) {
  cosine_partial_kernel<<<kCosineBlocks, 256, 0, st>>>(x, y, n, partials);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  cosine_final_kernel<<<1, 64, 0, st>>>(partials, out);
  return hipGetLastError();
}
hipError_t launch_summaries(const SummaryArgs& a, hipStream_t st) {
  if (!a.first_reject && !a.logp_mean && !a.loss_share) return hipSuccess;
  summary_rollout_kernel<<<(unsigned)a.B, 256, 0, st>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.logp_mean || a.loss_share) {
    summary_batch_kernel<<<1, 64, 0, st>>>(a);
    e = hipGetLastError();
  }
  return e;
}
hipError_t launch_candidate_audit(const CandArgs& a, hipStream_t st) {
  if (a.K <= 0) return hipSuccess;
  cand_pool_kernel<<<dim3((unsigned)(a.K * a.B), (unsigned)((a.H + 255) / 256)), 256, 0, st>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  cand_align_kernel<<<(unsigned)(a.K * a.B), 256, 0, st>>>(a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  cand_batch_kernel<<<(unsigned)a.K, 256, 0, st>>>(a);
  return hipGetLastError();
}
hipError_t launch_build_rows(const DevicePlan& pl, int32_t B, int64_t n_rows, int64_t n_pad,
                             hipStream_t st) {
  if (n_rows <= 0) return hipSuccess;
  const unsigned g = (unsigned)((n_pad + 255) / 256);
  build_rows_kernel<<<g, 256, 0, st>>>(pl, B, n_rows, n_pad);
  return hipGetLastError();
}
hipError_t launch_fill_f32(float* p, int64_t n, float v, hipStream_t st) {
  if (!p || n <= 0) return hipSuccess;
  fill_f32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(p, n, v);
  return hipGetLastError();
}
hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t st) {
  if (!p || n <= 0) return hipSuccess;
  fill_u32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(p, n, v);
  return hipGetLastError();
}

// Host -> device upload of a small blob through kernel arguments: the launch takes its copy
// of the bytes before it returns, so the host buffer may be pageable and may be freed or
// reused at once, whatever the stream still has to do, and the launch is an ordinary kernel
// node for a caller who captures the stream.
constexpr int kUploadChunk = 3072;   // bytes per launch (the argument block stays below 4 KiB)
struct UploadArgs { uint4* dst; int n16; uint4 data[kUploadChunk / 16]; };
__global__ __launch_bounds__(256) void upload_kernel(const UploadArgs a) {
  const int q = threadIdx.x;
  if (q < a.n16) a.dst[q] = a.data[q];
}
hipError_t launch_upload(void* dst, const void* src_host, size_t bytes, hipStream_t st) {
  if (bytes == 0) return hipSuccess;
  if (!dst || !src_host || (bytes & 15) || ((uintptr_t)dst & 15)) return hipErrorInvalidValue;
  static_assert(kUploadChunk / 16 <= 256, "one thread per 16 bytes");
  UploadArgs a;
  for (size_t at = 0; at < bytes; at += kUploadChunk) {
    const size_t nb = bytes - at < (size_t)kUploadChunk ? bytes - at : (size_t)kUploadChunk;
    a.dst = (uint4*)((unsigned char*)dst + at);
    a.n16 = (int)(nb / 16);
    memcpy(a.data, (const unsigned char*)src_host + at, nb);
    upload_kernel<<<1, 256, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}
hipError_t launch_segment_sums(const DevicePlan& pl, int32_t B, int probe, const float* klr,
                               const float* rownorm, double* seg, float* loss_prefix,
                               float* loss_full, hipStream_t st) {
  segment_sums_kernel<<<(unsigned)B, 256, 0, st>>>(pl, probe, klr, rownorm, seg, loss_prefix,
                                                   loss_full);
  return hipGetLastError();
}
hipError_t launch_alignment_and_batch(const BatchArgs& a, hipStream_t st) {
  rollout_alignment_kernel<<<(unsigned)a.B, 256, 0, st>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  batch_kernel<<<1, 256, 0, st>>>(a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// phase timer
// ---------------------------------------------------------------------------------------
PhaseTimer::~PhaseTimer() {
  for (auto& s : spans_) {
    if (s.a) (void)hipEventDestroy(s.a);
    if (s.b) (void)hipEventDestroy(s.b);
  }
}
void PhaseTimer::begin(int phase) {
  open_ = false;
  if (err_ != hipSuccess) return;
  Span s{phase, nullptr, nullptr};
  err_ = hipEventCreate(&s.a);
  if (err_ != hipSuccess) return;
  err_ = hipEventCreate(&s.b);
  if (err_ != hipSuccess) { (void)hipEventDestroy(s.a); return; }
  spans_.push_back(s);
  err_ = hipEventRecord(s.a, st_);
  open_ = err_ == hipSuccess;
}
void PhaseTimer::end() {
  if (!open_) return;
  open_ = false;
  err_ = hipEventRecord(spans_.back().b, st_);
}
hipError_t PhaseTimer::collect(float* phase_ms, int n_phases) {
  if (err_ != hipSuccess) return err_;
  hipError_t e = hipStreamSynchronize(st_);
  if (e != hipSuccess) return e;
  for (int k = 0; k < n_phases; ++k) phase_ms[k] = 0.f;
  for (auto& s : spans_) {
    float ms = 0.f;
    e = hipEventElapsedTime(&ms, s.a, s.b);
    if (e != hipSuccess) return e;
    if (s.phase >= 0 && s.phase < n_phases) phase_ms[s.phase] += ms;
  }
  return hipSuccess;
}

}  // namespace adwin
