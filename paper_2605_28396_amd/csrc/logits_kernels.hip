// Logits-given path: full-vocabulary log-softmax of student and teacher, per-token
// reverse KL (Eq. 2 at token level), sampled cost c_t (Sec. 2.3) and the logit gradient
// p_s((z_s - z_t) - mu) (Eq. 4 in expectation, App. A.1) on the admitted rows
// (Sec. 4.1), streamed from HBM.  One workgroup per packed row; two sweeps over the row.
#include <mutex>
#include <utility>
#include <vector>

#include "device_utils.h"
#include "plan_device.h"

namespace adwin {

constexpr int kRowThreads = 512;

struct LogitsArgs {
  DevicePlan pl;
  int32_t B, V;
  const uint4* z_s;
  const uint4* z_t;
  const int32_t* ids;
  float grad_scale;
  float* kl;
  float* c;
  uint4* dz;
  float* klr;          // [T] workspace copy of KL_t on computed rows (compact index)
  uint32_t* status;
  // teacher-side diagnostics (Sec. 3.1), each may be NULL
  float* t_logp; float* t_entropy; int32_t* t_rank;
  int sampled;         // dz = scale c_t (e_y - p_s) (Eq. 4 on the sampled token) instead of scale p_s (Delta - KL_t)
};

// The one-hot part of the sampled estimator: dz[y] = k (1 - p_s(y)), k = scale c_t, written
// over the -k p_s(y) the vector sweep stored there.
__device__ __forceinline__ void store_onehot(uint4* dzr, int y, float k, float zy_s, float lse_s) {
  const float v = k * (1.f - __expf(zy_s - lse_s));
  ((uint16_t*)dzr)[y] = (uint16_t)(pack_bf16(v, 0.f) & 0xffffu);
}

__device__ __forceinline__ void unpack8(const uint4& q, float (&f)[8]) {
  f[0] = bf16_lo(q.x); f[1] = bf16_hi(q.x);
  f[2] = bf16_lo(q.y); f[3] = bf16_hi(q.y);
  f[4] = bf16_lo(q.z); f[5] = bf16_hi(q.z);
  f[6] = bf16_lo(q.w); f[7] = bf16_hi(q.w);
}

// DIAG: also the teacher-side drift diagnostics of Sec. 3.1 for the row: entropy of the
// teacher distribution (H = lse_t - E_{p_t}[z_t]; the branching factor is exp(H)), the rank of
// y_t under the teacher (1 + number of entries with a strictly larger logit) and log p_t(y_t).
template <bool DIAG>
__global__ __launch_bounds__(kRowThreads) void logits_row_kernel(LogitsArgs a) {
  __shared__ float sh[7][kRowThreads / 64];
  __shared__ float bc[5];
  const int64_t t = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int nvec = a.V >> 3;
  const int i = last_le<int64_t>(a.pl.offsets, a.B + 1, t);
  const int64_t j = t - a.pl.offsets[i];
  uint4* dzr = a.dz ? a.dz + t * nvec : nullptr;
  if (j >= a.pl.n[i]) {   // outside the window: zero gradient row, zero KL
    if (dzr) {
      const uint4 z = {0u, 0u, 0u, 0u};
      for (int q = tid; q < nvec; q += kRowThreads) store16(dzr + q, z);
    }
    if (tid == 0) {
      if (a.kl) a.kl[t] = 0.f;
      if (a.c) a.c[t] = 0.f;
      if (DIAG) {
        if (a.t_logp) a.t_logp[t] = 0.f;
        if (a.t_entropy) a.t_entropy[t] = 0.f;
        if (a.t_rank) a.t_rank[t] = 0;
      }
    }
    return;
  }
  const uint4* zs = a.z_s + t * nvec;
  const uint4* zt = a.z_t + t * nvec;
  // sampled token and its teacher logit, for the rank
  int y = -1;
  float zy_rank = 0.f;
  if (DIAG && a.ids) {
    y = a.ids[t];
    if (y >= 0 && y < a.V) zy_rank = __uint_as_float((uint32_t)((const uint16_t*)zt)[y] << 16);
    else y = -1;
  }
  float Bt = 0.f;     // sum e^{z_t - m_t} z_t
  int cnt = 0;        // entries the teacher ranks strictly above y_t

  // ---- sweep 1: running max / sum-exp of both rows and A = sum e^{z_s-m}(z_s-z_t) ----
  float ms = kNegBig, Zs = 0.f, A = 0.f, mt = kNegBig, Zt = 0.f;
  for (int q = tid; q < nvec; q += kRowThreads) {
    const uint4 qs = zs[q], qt = zt[q];
    float s[8], u[8];
    unpack8(qs, s);
    unpack8(qt, u);
    float mx = s[0], mxt = u[0];
#pragma unroll
    for (int k = 1; k < 8; ++k) { mx = fmaxf(mx, s[k]); mxt = fmaxf(mxt, u[k]); }
    if (mx > ms) {
      const float sc = fast_exp2((ms - mx) * kLog2e);
      Zs *= sc; A *= sc; ms = mx;
    }
    if (mxt > mt) {
      const float sc = fast_exp2((mt - mxt) * kLog2e);
      Zt *= sc; Bt *= sc; mt = mxt;
    }
    const float ms2 = ms * kLog2e, mt2 = mt * kLog2e;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const float e = fast_exp2(fmaf(s[k], kLog2e, -ms2));
      Zs += e;
      A = fmaf(e, s[k] - u[k], A);
      const float et = fast_exp2(fmaf(u[k], kLog2e, -mt2));
      Zt += et;
      if (DIAG) {
        Bt = fmaf(et, u[k], Bt);
        cnt += (u[k] > zy_rank && q * 8 + k != y) ? 1 : 0;
      }
    }
  }
  // wave then block merge, fixed order
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    merge_mza(ms, Zs, A, __shfl_xor(ms, o, 64), __shfl_xor(Zs, o, 64), __shfl_xor(A, o, 64));
    if (DIAG) {
      merge_mza(mt, Zt, Bt, __shfl_xor(mt, o, 64), __shfl_xor(Zt, o, 64), __shfl_xor(Bt, o, 64));
      cnt += __shfl_xor(cnt, o, 64);
    } else {
      merge_mz(mt, Zt, __shfl_xor(mt, o, 64), __shfl_xor(Zt, o, 64));
    }
  }
  if (lane == 0) {
    sh[0][w] = ms; sh[1][w] = Zs; sh[2][w] = A; sh[3][w] = mt; sh[4][w] = Zt;
    if (DIAG) { sh[5][w] = Bt; sh[6][w] = __int_as_float(cnt); }
  }
  __syncthreads();
  if (tid == 0) {
    float m = sh[0][0], Z = sh[1][0], Aa = sh[2][0], m2 = sh[3][0], Z2 = sh[4][0];
    float B2 = DIAG ? sh[5][0] : 0.f;
    int rank = DIAG ? __float_as_int(sh[6][0]) : 0;
    for (int k = 1; k < kRowThreads / 64; ++k) {
      merge_mza(m, Z, Aa, sh[0][k], sh[1][k], sh[2][k]);
      if (DIAG) {
        merge_mza(m2, Z2, B2, sh[3][k], sh[4][k], sh[5][k]);
        rank += __float_as_int(sh[6][k]);
      } else {
        merge_mz(m2, Z2, sh[3][k], sh[4][k]);
      }
    }
    const float lse_s = m + logf(Z), lse_t = m2 + logf(Z2);
    const float mu = Aa / Z;                       // E_{p_s}[z_s - z_t]
    float kl = kl_from_sums(mu, m - m2, Z, Z2);
    float ent = DIAG ? lse_t - B2 / Z2 : 0.f;
    // a row without finite statistics is excluded: zeros in every output
    const bool dead = !(fabsf(lse_s) < 3.0e38f) || !(fabsf(lse_t) < 3.0e38f) || !(fabsf(kl) < 3.0e38f) ||
                      !(fabsf(mu) < 3.0e38f) || !(fabsf(ent) < 3.0e38f);
    float c = 0.f;
    uint32_t flag = dead ? ADWIN_DEV_NONFINITE : 0u;
    if (dead) { kl = 0.f; ent = 0.f; }
    if (a.ids && !dead) {
      const int y = a.ids[t];
      if (y >= 0 && y < a.V) {
        const uint16_t* ps = (const uint16_t*)zs;
        const uint16_t* pt = (const uint16_t*)zt;
        const float zy_s = __uint_as_float((uint32_t)ps[y] << 16);
        const float zy_t = __uint_as_float((uint32_t)pt[y] << 16);
        c = (zy_s - lse_s) - (zy_t - lse_t);
      } else {
        flag |= ADWIN_DEV_BAD_ID;
      }
    }
    if (flag && a.status) atomicOr(a.status, flag);
    if (a.kl) a.kl[t] = kl;
    if (a.c) a.c[t] = c;
    if (DIAG) {
      if (a.t_entropy) a.t_entropy[t] = ent;
      if (a.t_logp) a.t_logp[t] = (y >= 0 && !dead) ? zy_rank - lse_t : 0.f;
      if (a.t_rank) a.t_rank[t] = (y >= 0 && !dead) ? rank + 1 : 0;
    }
    a.klr[a.pl.comp_off[i] + j] = kl;
    bc[0] = lse_s * kLog2e;
    bc[1] = mu;
    bc[2] = c;
    bc[3] = lse_s;
    bc[4] = dead ? 1.f : 0.f;
  }
  __syncthreads();
  if (!dzr) return;
  if (bc[4] != 0.f) {
    const uint4 z = {0u, 0u, 0u, 0u};
    for (int q = tid; q < nvec; q += kRowThreads) store16(dzr + q, z);
    return;
  }
  // ---- sweep 2: dz = scale * p_s * ((z_s - z_t) - mu), or scale * c_t * (e_y - p_s) ---
  const float lse2 = bc[0];
  const float scale = a.grad_scale * a.pl.alpha_p[i];
  const float ca = a.sampled ? 0.f : 1.f, cb = a.sampled ? -bc[2] : -bc[1];
  for (int q = tid; q < nvec; q += kRowThreads) {
    const uint4 qs = zs[q], qt = zt[q];
    float s[8], u[8], d[8];
    unpack8(qs, s);
    unpack8(qt, u);
#pragma unroll
    for (int k = 0; k < 8; ++k)
      d[k] = scale * fast_exp2(fmaf(s[k], kLog2e, -lse2)) * fmaf(s[k] - u[k], ca, cb);
    uint4 o;
    o.x = pack_bf16(d[0], d[1]);
    o.y = pack_bf16(d[2], d[3]);
    o.z = pack_bf16(d[4], d[5]);
    o.w = pack_bf16(d[6], d[7]);
    store16(dzr + q, o);
  }
  if (a.sampled) {
    __syncthreads();
    if (tid == 0 && a.ids) {
      const int yy = a.ids[t];
      if (yy >= 0 && yy < a.V)
        store_onehot(dzr, yy, scale * bc[2], __uint_as_float((uint32_t)((const uint16_t*)zs)[yy] << 16), bc[3]);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Row-resident variant.  One 256-thread workgroup (one wave per SIMD, up to 512 registers
// per lane) per packed row keeps the whole row pair on chip between the two sweeps: z_s in
// registers, z_t partly in LDS and partly in registers, so HBM sees each logit once
// (4 B read + 2 B written per element).  Rows longer than kResVec vectors re-read the
// excess from memory.
// ---------------------------------------------------------------------------------------
constexpr int kResThreads = 256;
constexpr int kResIters = 75;                      // vectors of 8 logits per thread
constexpr int kResTLds = 39;                       // of which z_t vectors parked in LDS
constexpr int kResTReg = kResIters - kResTLds;     // and in registers
constexpr int kResBatch = 5;                       // iterations whose loads are issued together
constexpr int kResDepth = 1;                       // batches in flight ahead of the arithmetic (2 and 3: no faster)
constexpr int kResVec = kResIters * kResThreads;   // 19,200 vectors = 153,600 logits
constexpr int kResLdsBytes = kResTLds * kResThreads * 16 + 256;

template <int... I, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
// Calls f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index
// is a compile-time constant, so that register arrays are never indexed dynamically.
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// Row access through buffer descriptors: base = the row, extent = its bytes.  Every 16-byte
// access is then one instruction with a lane offset shared by all of them (16 * thread index)
// and a scalar offset per iteration, no 64-bit address per access to compute or to keep in
// vector registers (with 150 accesses per sweep those addresses, computed ahead by the
// compiler, crowded the row itself out of the register file); an access beyond the extent reads
// zeros / is dropped by the hardware, which is what the ragged last iteration needs.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t row_rsrc(const void* row, int bytes) {
  // flag word: the raw-buffer setting of the gfx9 family (32-bit data format, no swizzle)
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(row), 0, bytes, 0x00020000);
}
__device__ __forceinline__ uint4 row_load16(__amdgpu_buffer_rsrc_t r, int lane_off, int iter_off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, iter_off, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void row_store16(__amdgpu_buffer_rsrc_t r, int lane_off, int iter_off, const uint4& v) {
  u32x4 x;
  x.x = v.x; x.y = v.y; x.z = v.z; x.w = v.w;
  __builtin_amdgcn_raw_buffer_store_b128(x, r, lane_off, iter_off, 0);
}

struct RowStats { float ms, Zs, A, mt, Zt; };

__device__ __forceinline__ float max8(const float (&v)[8]) {
  return fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
}

__device__ __forceinline__ void stats_update(RowStats& r, const uint4& qs, const uint4& qt) {
  float s[8], u[8];
  unpack8(qs, s);
  unpack8(qt, u);
  const float mx = max8(s), mxt = max8(u);
  if (mx > r.ms) {
    const float sc = fast_exp2((r.ms - mx) * kLog2e);
    r.Zs *= sc; r.A *= sc; r.ms = mx;
  }
  if (mxt > r.mt) { r.Zt *= fast_exp2((r.mt - mxt) * kLog2e); r.mt = mxt; }
  const float ms2 = r.ms * kLog2e, mt2 = r.mt * kLog2e;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const float e = fast_exp2(fmaf(s[k], kLog2e, -ms2));
    r.Zs += e;
    r.A = fmaf(e, s[k] - u[k], r.A);
    r.Zt += fast_exp2(fmaf(u[k], kLog2e, -mt2));
  }
}

// dz = sgn * 2^(z_s*log2e - lse2s) * ((z_s - z_t) - mu), with |scale| folded into lse2s
__device__ __forceinline__ uint4 dz_vector(const uint4& qs, const uint4& qt, float lse2s, float sgn,
                                           float neg_sgn_mu) {
  float s[8], u[8], d[8];
  unpack8(qs, s);
  unpack8(qt, u);
#pragma unroll
  for (int k = 0; k < 8; ++k)
    d[k] = fast_exp2(fmaf(s[k], kLog2e, -lse2s)) * fmaf(s[k] - u[k], sgn, neg_sgn_mu);
  uint4 o;
  o.x = pack_bf16(d[0], d[1]);
  o.y = pack_bf16(d[2], d[3]);
  o.z = pack_bf16(d[4], d[5]);
  o.w = pack_bf16(d[6], d[7]);
  return o;
}

__global__ __launch_bounds__(kResThreads, 1) void logits_row_resident_kernel(LogitsArgs a) {
  extern __shared__ __align__(16) char lds_raw[];
  uint4* lds_t = (uint4*)lds_raw;
  float* sh = (float*)(lds_raw + kResTLds * kResThreads * 16);   // [5][4] + broadcast [5]
  const int64_t t = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int nvec = a.V >> 3;
  const int i = last_le<int64_t>(a.pl.offsets, a.B + 1, t);
  const int64_t j = t - a.pl.offsets[i];
  uint4* dzr = a.dz ? a.dz + t * nvec : nullptr;
  if (j >= a.pl.n[i]) {
    if (dzr) {
      const uint4 z = {0u, 0u, 0u, 0u};
      for (int q = tid; q < nvec; q += kResThreads) store16(dzr + q, z);
    }
    if (tid == 0) {
      if (a.kl) a.kl[t] = 0.f;
      if (a.c) a.c[t] = 0.f;
    }
    return;
  }
  const uint4* zs = a.z_s + t * nvec;
  const uint4* zt = a.z_t + t * nvec;
  // bf16 -3.39e38 in every lane: neutral for max, exp and the difference
  const uint4 neutral = {0xff7fff7fu, 0xff7fff7fu, 0xff7fff7fu, 0xff7fff7fu};

  uint4 rs[kResIters];
  uint4 rt[kResTReg];
  RowStats st = {kNegBig, 0.f, 0.f, kNegBig, 0.f};
  // ---- sweep 1: load the row pair once, keep it, accumulate the statistics ------------
  // Loads are issued kResDepth batches (of kResBatch iterations) ahead of the arithmetic, so
  // that the single wave per SIMD always has 2 * kResBatch 16-byte loads in flight per lane.
  // z_s vectors and the register-resident z_t vectors land in their final registers (the
  // loads write accumulation registers directly); the z_t vectors that go to the LDS pass
  // through a small staging ring.  Lanes beyond the row read zeros and take a neutral value.
  const int row_bytes = nvec * 16, lane_off = tid * 16;
  const __amdgpu_buffer_rsrc_t bs = row_rsrc(zs, row_bytes), bt = row_rsrc(zt, row_bytes);
  uint4 tb[kResDepth + 1][kResBatch];
  auto issue = [&](auto b_c) {
    constexpr int b = decltype(b_c)::value;
    if constexpr (b < kResIters / kResBatch) {
      static_for<kResBatch>([&](auto g_c) {
        constexpr int g = decltype(g_c)::value;
        constexpr int it = b * kResBatch + g;
        rs[it] = row_load16(bs, lane_off, it * kResThreads * 16);
        if constexpr (it < kResTLds) tb[b % (kResDepth + 1)][g] = row_load16(bt, lane_off, it * kResThreads * 16);
        else rt[it - kResTLds] = row_load16(bt, lane_off, it * kResThreads * 16);
      });
    }
  };
  static_for<kResDepth>([&](auto b_c) { issue(b_c); });
  static_for<kResIters / kResBatch>([&](auto b_c) {
    constexpr int b = decltype(b_c)::value;
    issue(std::integral_constant<int, b + kResDepth>{});
    if (b * kResBatch * kResThreads < nvec) {
      static_for<kResBatch>([&](auto g_c) {
        constexpr int g = decltype(g_c)::value;
        constexpr int it = b * kResBatch + g;
        const bool in = it * kResThreads + tid < nvec;
        uint4 qs = rs[it], qt;
        if constexpr (it < kResTLds) qt = tb[b % (kResDepth + 1)][g]; else qt = rt[it - kResTLds];
        if (!in) { qs = neutral; qt = neutral; }
        if constexpr (it < kResTLds) lds_t[it * kResThreads + tid] = qt;
        stats_update(st, qs, qt);
      });
    }
  });
  for (int q = kResVec + tid; q < nvec; q += kResThreads) stats_update(st, zs[q], zt[q]);
  float Zs = st.Zs, As = st.A, Zt = st.Zt;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    merge_mza(st.ms, Zs, As, __shfl_xor(st.ms, o, 64), __shfl_xor(Zs, o, 64), __shfl_xor(As, o, 64));
    merge_mz(st.mt, Zt, __shfl_xor(st.mt, o, 64), __shfl_xor(Zt, o, 64));
  }
  if (lane == 0) { sh[0 + w] = st.ms; sh[4 + w] = Zs; sh[8 + w] = As; sh[12 + w] = st.mt; sh[16 + w] = Zt; }
  __syncthreads();
  if (tid == 0) {
    float m = sh[0], Z = sh[4], Aa = sh[8], m2 = sh[12], Z2 = sh[16];
    for (int k = 1; k < kResThreads / 64; ++k) {
      merge_mza(m, Z, Aa, sh[k], sh[4 + k], sh[8 + k]);
      merge_mz(m2, Z2, sh[12 + k], sh[16 + k]);
    }
    const float lse_s = m + logf(Z), lse_t = m2 + logf(Z2);
    const float mu = Aa / Z;                       // E_{p_s}[z_s - z_t]
    float kl = kl_from_sums(mu, m - m2, Z, Z2);
    // a row without finite statistics is excluded: zeros in every output
    const bool dead = !(fabsf(lse_s) < 3.0e38f) || !(fabsf(lse_t) < 3.0e38f) || !(fabsf(kl) < 3.0e38f) ||
                      !(fabsf(mu) < 3.0e38f);
    float c = 0.f;
    uint32_t flag = dead ? ADWIN_DEV_NONFINITE : 0u;
    if (dead) kl = 0.f;
    if (a.ids && !dead) {
      const int y = a.ids[t];
      if (y >= 0 && y < a.V) {
        const float zy_s = __uint_as_float((uint32_t)((const uint16_t*)zs)[y] << 16);
        const float zy_t = __uint_as_float((uint32_t)((const uint16_t*)zt)[y] << 16);
        c = (zy_s - lse_s) - (zy_t - lse_t);
      } else {
        flag |= ADWIN_DEV_BAD_ID;
      }
    }
    if (flag && a.status) atomicOr(a.status, flag);
    if (a.kl) a.kl[t] = kl;
    if (a.c) a.c[t] = c;
    a.klr[a.pl.comp_off[i] + j] = kl;
    sh[20] = lse_s * kLog2e;
    sh[21] = mu;
    sh[22] = c;
    sh[23] = lse_s;
    sh[24] = dead ? 1.f : 0.f;
  }
  __syncthreads();
  if (!dzr) return;
  if (sh[24] != 0.f) {
    const uint4 z = {0u, 0u, 0u, 0u};
    for (int q = tid; q < nvec; q += kResThreads) store16(dzr + q, z);
    return;
  }
  // ---- sweep 2: dz from the resident copy ----------------------------------------------
  // expected: scale p_s ((z_s - z_t) - mu); sampled: -k p_s with k = scale c_t (the one-hot
  // term follows); |scale| resp. |k| is folded into the exponent, the sign into the factor
  const float scale = a.grad_scale * a.pl.alpha_p[i];
  const float k_s = a.sampled ? scale * sh[22] : scale;
  const float sg = k_s < 0.f ? -1.f : 1.f;
  const float sgn = a.sampled ? 0.f : sg;
  const float lse2 = sh[20] - log2f(fabsf(k_s)), nmu = a.sampled ? -sg : -sg * sh[21];
  const __amdgpu_buffer_rsrc_t bd = row_rsrc(dzr, row_bytes);
  static_for<kResIters>([&](auto it_c) {
    constexpr int it = decltype(it_c)::value;
    if (it * kResThreads < nvec) {
      uint4 qt;
      if constexpr (it < kResTLds) qt = lds_t[it * kResThreads + tid]; else qt = rt[it - kResTLds];
      row_store16(bd, lane_off, it * kResThreads * 16, dz_vector(rs[it], qt, lse2, sgn, nmu));
    }
  });
  for (int q = kResVec + tid; q < nvec; q += kResThreads)
    store16(dzr + q, dz_vector(zs[q], zt[q], lse2, sgn, nmu));
  if (a.sampled) {
    __syncthreads();
    if (tid == 0 && a.ids) {
      const int yy = a.ids[t];
      if (yy >= 0 && yy < a.V)
        store_onehot(dzr, yy, k_s, __uint_as_float((uint32_t)((const uint16_t*)zs)[yy] << 16), sh[23]);
    }
  }
}

hipError_t logits_kernels_opt_in() {
  return hipFuncSetAttribute((const void*)logits_row_resident_kernel,
                             hipFuncAttributeMaxDynamicSharedMemorySize, kResLdsBytes);
}

struct LogitsLayout {
  size_t o_plan, o_klr, o_seg, o_racc, o_summ, total;
  LogitsLayout(int32_t B, int64_t T) {
    size_t o = 0;
    o_plan = o; o += PlanBlobLayout(B).bytes;
    o_klr = o;  o = align_up(o + sizeof(float) * (size_t)(T > 0 ? T : 1), 256);
    o_seg = o;  o = align_up(o + sizeof(double) * 4 * (size_t)B, 256);
    o_racc = o; o = align_up(o + sizeof(double) * 4 * (size_t)B, 256);
    o_summ = o; o = align_up(o + sizeof(double) * kSummarySlots * (size_t)B, 256);
    total = o;
  }
};

static int check_logits_problem(const adwin_opd_logits_problem* p) {
  if (!p) return ADWIN_E_NULL;
  if (p->struct_bytes != sizeof(adwin_opd_logits_problem)) return ADWIN_E_MODE;
  int st = validate_ragged(p->T, p->B, p->offsets, p->window);
  if (st != ADWIN_OK) return st;
  if (p->V <= 0 || (p->V & 7)) return ADWIN_E_SHAPE;
  if (p->reduction < ADWIN_RED_SEQ_MEAN || p->reduction > ADWIN_RED_TOKEN_MEAN) return ADWIN_E_MODE;
  if (p->estimator != ADWIN_EST_EXPECTED && p->estimator != ADWIN_EST_SAMPLED) return ADWIN_E_MODE;
  if (p->estimator == ADWIN_EST_SAMPLED && !p->ids) return ADWIN_E_NULL;
  if (p->scheme < ADWIN_LOGITS_AUTO || p->scheme > ADWIN_LOGITS_STREAMING) return ADWIN_E_MODE;
  if (p->t_first_reject && !p->t_rank) return ADWIN_E_NULL;
  if (p->t_first_reject && p->topk <= 0) return ADWIN_E_SHAPE;
  if (p->t_logp_mean && !p->t_logp) return ADWIN_E_NULL;
  return ADWIN_OK;
}

}  // namespace adwin

using namespace adwin;

extern "C" int adwin_opd_logits_workspace_bytes(const adwin_opd_logits_problem* p, size_t* bytes) {
  if (!bytes) return ADWIN_E_NULL;
  int st = check_logits_problem(p);
  if (st != ADWIN_OK) return st;
  *bytes = LogitsLayout(p->B, p->T).total;
  return ADWIN_OK;
}

static int logits_impl(const adwin_opd_logits_problem* p, void* workspace, size_t workspace_bytes,
                       void* hip_stream, PhaseTimer* timer) {
  int st = check_logits_problem(p);
  if (st != ADWIN_OK) return st;
  if (p->T > 0 && (!p->z_s || !p->z_t)) return ADWIN_E_NULL;
  const uintptr_t al = (uintptr_t)p->z_s | (uintptr_t)p->z_t | (uintptr_t)p->dz;
  if (al & 15) return ADWIN_E_ALIGN;
  LogitsLayout L(p->B, p->T);
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < L.total)
    return ADWIN_E_WORKSPACE;
  hipStream_t stream = (hipStream_t)hip_stream;
  unsigned char* ws = (unsigned char*)workspace;

  std::vector<unsigned char> blob;
  HostPlan hp = make_host_plan(p->T, p->B, p->offsets, p->window, /*probe=*/0, p->reduction, &blob);
  ADWIN_HIP_TRY(launch_upload(ws + L.o_plan, blob.data(), blob.size(), stream));
  DevicePlan pl = device_plan_at(ws + L.o_plan, p->B, nullptr, nullptr);
  float* klr = (float*)(ws + L.o_klr);
  double* seg = (double*)(ws + L.o_seg);

  ADWIN_HIP_TRY(launch_fill_u32(p->status_dev, 1, 0u, stream));
  if (p->T > 0) {
    LogitsArgs a;
    a.pl = pl; a.B = p->B; a.V = p->V;
    a.z_s = (const uint4*)p->z_s; a.z_t = (const uint4*)p->z_t; a.ids = p->ids;
    a.grad_scale = p->grad_scale;
    a.kl = p->kl; a.c = p->c; a.dz = (uint4*)p->dz; a.klr = klr; a.status = p->status_dev;
    a.t_logp = p->t_logp; a.t_entropy = p->t_entropy; a.t_rank = p->t_rank;
    a.sampled = p->estimator == ADWIN_EST_SAMPLED;
    PhaseScope scope(timer, ADWIN_PHASE_STATS);
    const bool streaming = p->scheme == ADWIN_LOGITS_STREAMING;
    if (p->t_logp || p->t_entropy || p->t_rank) {
      // the diagnostics ride on the streaming kernel (the row-resident one has no register to spare)
      logits_row_kernel<true><<<(unsigned)p->T, kRowThreads, 0, stream>>>(a);
    } else if (streaming) {
      logits_row_kernel<false><<<(unsigned)p->T, kRowThreads, 0, stream>>>(a);
    } else {
      if (first_use_on_device(1)) ADWIN_HIP_TRY(logits_kernels_opt_in());
      logits_row_resident_kernel<<<(unsigned)p->T, kResThreads, kResLdsBytes, stream>>>(a);
    }
    ADWIN_HIP_TRY(hipGetLastError());
  }
  PhaseScope scope(timer, ADWIN_PHASE_REDUCE);
  ADWIN_HIP_TRY(launch_segment_sums(pl, p->B, 0, klr, nullptr, seg, p->loss_prefix, nullptr, stream));
  BatchArgs b{};
  b.pl = pl; b.B = p->B; b.H = 0; b.probe = 0; b.zero_grad = 1; b.seg = seg;
  b.up = nullptr; b.uf = nullptr; b.racc = (double*)(ws + L.o_racc);
  b.rho_pooled = nullptr; b.rho_field = nullptr; b.batch = p->batch;
  b.n_out = p->n_out; b.n_adm_out = p->n_adm_out; b.n_adm = hp.n_adm;
  ADWIN_HIP_TRY(launch_alignment_and_batch(b, stream));
  if (p->t_first_reject || p->t_logp_mean) {
    SummaryArgs sa{};
    sa.pl = pl; sa.B = p->B; sa.probe = 0; sa.topk = p->topk; sa.K = 0;
    sa.t_rank = p->t_rank; sa.t_logp = p->t_logp; sa.kl = nullptr;
    sa.acc = (double*)(ws + L.o_summ);
    sa.first_reject = p->t_first_reject; sa.logp_mean = p->t_logp_mean; sa.loss_share = nullptr;
    ADWIN_HIP_TRY(launch_summaries(sa, stream));
  }
  return ADWIN_OK;
}

extern "C" int adwin_opd_from_logits(const adwin_opd_logits_problem* p, void* workspace,
                                     size_t workspace_bytes, void* hip_stream) {
  return logits_impl(p, workspace, workspace_bytes, hip_stream, nullptr);
}

// ---------------------------------------------------------------------------------------
// The entry point that allocates nothing: the same call with its scratch (plan blob,
// per-row KL copy, per-rollout accumulators) in a fixed array inside the library.  Every GPU
// holds its own copy of the array at its own address; the name `static_scratch` is only the
// host-side handle of the symbol, so host code asks the runtime for the device address once per
// device and uses that pointer from then on.  (No `used` attribute on the array: the compiler
// makes a file-local device variable visible to the runtime's lookup by name only because host
// code refers to it, and that attribute switches this off.)
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char static_scratch[ADWIN_STATIC_SCRATCH_BYTES];

namespace adwin {

static std::mutex g_static_mu;
static void* g_static_ptr[64];          // device address of static_scratch, per device ordinal

// Address of the current device's copy of static_scratch (looked up on first use per device).
static hipError_t static_scratch_ptr(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(static_scratch));
    if (e != hipSuccess) return e;
    if (!ptr || ((uintptr_t)ptr & 255)) return hipErrorInvalidSymbol;
    g_static_ptr[dev] = ptr;
  }
  *out = g_static_ptr[dev];
  return hipSuccess;
}

hipError_t logits_static_setup() {
  void* ptr = nullptr;
  return static_scratch_ptr(&ptr);
}

}  // namespace adwin

extern "C" int adwin_opd_from_logits_static(const adwin_opd_logits_problem* p, void* hip_stream) {
  int st = check_logits_problem(p);
  if (st != ADWIN_OK) return st;
  if (LogitsLayout(p->B, p->T).total > (size_t)ADWIN_STATIC_SCRATCH_BYTES) return ADWIN_E_WORKSPACE;
  void* ptr = nullptr;
  ADWIN_HIP_TRY(static_scratch_ptr(&ptr));
  // Nothing in the scratch has to start at zero: every kernel of the call writes what a later
  // one reads (the plan blob, KL of every admitted row, the per-rollout sums), so what the
  // previous call left behind is never read.
  return logits_impl(p, ptr, (size_t)ADWIN_STATIC_SCRATCH_BYTES, hip_stream, nullptr);
}

extern "C" int adwin_opd_from_logits_profile(const adwin_opd_logits_problem* p, void* workspace,
                                             size_t workspace_bytes, void* hip_stream,
                                             float* phase_ms) {
  if (!phase_ms) return ADWIN_E_NULL;
  PhaseTimer timer((hipStream_t)hip_stream);
  int st = logits_impl(p, workspace, workspace_bytes, hip_stream, &timer);
  if (st != ADWIN_OK) return st;
  ADWIN_HIP_TRY(timer.collect(phase_ms, ADWIN_N_PHASES));
  return ADWIN_OK;
}
