// Fused path: LM-head projections on bf16 MFMA, full-vocabulary online log-sum-exp,
// per-token reverse KL (Eq. 2 at token level), logit gradient (Eq. 4 in expectation,
// App. A.1) and its contraction with W_s back to the student hidden state.
//
// Pass 1 (stats)  : for a 256-token tile, walk vocabulary tiles of 128; per tile two MFMA
//                   GEMMs (teacher, student) into fp32 accumulators, then an in-register
//                   online update of (m_s, Z_s, A = sum e^{z_s-m_s}(z_s-z_t), m_t, Z_t).
// Merge           : per row: lse_s, lse_t, mu = A/Z_s, KL_t = mu - lse_s + lse_t, c_t.
// Pass 2 (dz)     : same GEMMs again, dz = p_s((z_s-z_t) - mu) rounded to bf16 into a
//                   bounded row slab (never the logits, never a full [rows, V] array).
// Pass 3 (grad)   : g = dz W_s as an MFMA GEMM over the slab with k = vocabulary.
// Finalize        : scale by grad_scale*alpha, scatter to dh_prefix / dh_full, row norms.
//
// MFMA operand roles: v_mfma_f32_32x32x16_bf16 computes D[i][j] += sum_k A[i][k] B[k][j]
// with i in registers and j = lane % 32.  In the logit passes A = W tile (i = vocabulary)
// and B = h tile (j = token), so each lane owns one token column and the reduction over
// the vocabulary runs down its own registers with no cross-lane traffic.
#include <utility>
#include <vector>

#include "device_utils.h"
#include "plan_device.h"

namespace adwin {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kRowBytes = kBK * 2;   // 128 B of k per staged row

// ---------------------------------------------------------------------------------------
// Staging of [ROWS x 64] bf16 tiles: global -> registers -> LDS.  Thread t moves the
// 16-byte chunk (t & 7) of rows (t >> 3) + 32 i.  Chunk c of row r is stored at chunk
// position c ^ ((r >> 1) & 7): two 128-byte rows span all 64 LDS banks, so the 16 rows
// that 16 consecutive lanes of an MFMA fragment read touch land on 16 distinct
// (row parity, position) pairs, i.e. on distinct banks.
// ---------------------------------------------------------------------------------------
template <int ROWS>
struct RowStager {
  static constexpr int N = ROWS / 32;
  const uint4* p[N];
  uint4 v[N];
  __device__ __forceinline__ void issue(int kt) {
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = p[i][kt * 8];
  }
  __device__ __forceinline__ void commit(char* tile, int thread_off) const {
#pragma unroll
    for (int i = 0; i < N; ++i) *(uint4*)(tile + thread_off + i * 32 * kRowBytes) = v[i];
  }
};

__device__ __forceinline__ int stage_thread_off(int tid) {
  const int r = tid >> 3, c = tid & 7;
  return r * kRowBytes + ((c ^ ((r >> 1) & 7)) << 4);
}

// acc[FM][FN] += A_tile(wave rows) * B_tile(wave rows)^T for one staged k-step of 64.
template <int FM, int FN>
__device__ __forceinline__ void mma_stage(f32x16 (&acc)[FM][FN], const char* tA, const char* tB,
                                          int lane) {
  const int row_off = (lane & 31) * kRowBytes;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const int sw = ((kk * 2 + (lane >> 5)) ^ ((lane >> 1) & 7)) << 4;
    bf16x8 a[FM], b[FN];
#pragma unroll
    for (int fm = 0; fm < FM; ++fm)
      a[fm] = *(const bf16x8*)(tA + fm * 32 * kRowBytes + row_off + sw);
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
      b[fn] = *(const bf16x8*)(tB + fn * 32 * kRowBytes + row_off + sw);
#pragma unroll
    for (int fm = 0; fm < FM; ++fm)
#pragma unroll
      for (int fn = 0; fn < FN; ++fn)
        acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[fm], b[fn], acc[fm][fn], 0, 0, 0);
  }
}

// Double-buffered k loop.  ldsA/ldsB: stage 0 tiles; stage 1 follows at `stage_bytes`.
// waveA/waveB: byte offset of this wave's rows inside the A/B tile.
template <int RA, int RB, int FM, int FN>
__device__ __forceinline__ void gemm_kloop(f32x16 (&acc)[FM][FN], RowStager<RA>& sa,
                                           RowStager<RB>& sb, int kt0, int nk, char* lds,
                                           int stage_bytes, int waveA, int waveB, int tid) {
  constexpr int kOffB = RA * kRowBytes;
  const int toff = stage_thread_off(tid);
  const int lane = tid & 63;
  sa.issue(kt0);
  sb.issue(kt0);
  sa.commit(lds, toff);
  sb.commit(lds + kOffB, toff);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    char* cur = lds + (kt & 1) * stage_bytes;
    char* nxt = lds + ((kt + 1) & 1) * stage_bytes;
    const bool more = kt + 1 < nk;
    if (more) {
      sa.issue(kt0 + kt + 1);
      sb.issue(kt0 + kt + 1);
    }
    mma_stage<FM, FN>(acc, cur + waveA, cur + kOffB + waveB, lane);
    if (more) {
      sa.commit(nxt, toff);
      sb.commit(nxt + kOffB, toff);
    }
    __syncthreads();
  }
}

// Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
// virtual ids so that the tiles sharing operands also share an L2.
__device__ __forceinline__ int xcd_contiguous_id(int bid, int nb) {
  const int xcd = bid & 7, loc = bid >> 3;
  const int base = nb >> 3, rem = nb & 7;
  return xcd * base + (xcd < rem ? xcd : rem) + loc;
}

// ---------------------------------------------------------------------------------------
// Logit passes
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

// Running per-token statistics held by one lane for its two token columns.
struct LaneStats { float m_s[2], Z_s[2], A_s[2], m_t[2], Z_t[2]; };

// Element e of block fm sits at vocabulary row v0 + fm*32 + 8*(e/4) + 4*(lane/32) + e%4.
// Online update of (m_s, Z_s, A, m_t, Z_t) with one 128 x 64 logit tile per wave.
__device__ __forceinline__ void stats_epilogue(const f32x16 (&zs)[4][2], const f32x16 (&zt)[4][2],
                                               LaneStats& st, int v0, int V, bool tail, int lane) {
  const int vlane = v0 + 4 * (lane >> 5);
#pragma unroll
  for (int fn = 0; fn < 2; ++fn) {
    float mxs = st.m_s[fn], mxt = st.m_t[fn];
#pragma unroll
    for (int fm = 0; fm < 4; ++fm)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const bool ok = !tail || (vlane + fm * 32 + 8 * (e >> 2) + (e & 3)) < V;
        if (ok) { mxs = fmaxf(mxs, zs[fm][fn][e]); mxt = fmaxf(mxt, zt[fm][fn][e]); }
      }
    const float scs = fast_exp2((st.m_s[fn] - mxs) * kLog2e);
    const float sct = fast_exp2((st.m_t[fn] - mxt) * kLog2e);
    float Zs = st.Z_s[fn] * scs, As = st.A_s[fn] * scs, Zt = st.Z_t[fn] * sct;
    const float ms2 = mxs * kLog2e, mt2 = mxt * kLog2e;
#pragma unroll
    for (int fm = 0; fm < 4; ++fm)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const bool ok = !tail || (vlane + fm * 32 + 8 * (e >> 2) + (e & 3)) < V;
        const float s = zs[fm][fn][e], t = zt[fm][fn][e];
        float es = fast_exp2(fmaf(s, kLog2e, -ms2));
        float et = fast_exp2(fmaf(t, kLog2e, -mt2));
        float d = s - t;
        if (!ok) { es = 0.f; et = 0.f; d = 0.f; }
        Zs += es;
        As = fmaf(es, d, As);
        Zt += et;
      }
    st.m_s[fn] = mxs; st.m_t[fn] = mxt; st.Z_s[fn] = Zs; st.A_s[fn] = As; st.Z_t[fn] = Zt;
  }
}

// Slab layout (the A operand of the gradient GEMM, see "Tile images" below): block
// (row tile, k-step) of 256 rows x 64 vocabulary entries, row r at r * 64 elements, its
// 8-entry chunk c at chunk position c ^ ((r >> 1) & 7).  A 256 x 128 logit tile covers the
// two consecutive blocks 2 vt and 2 vt + 1 of its row tile; `blk` points at the first.
constexpr int kSlabBlock = kTileTokens * kBK;   // elements per block
constexpr int kImgBytesSlab = kSlabBlock * 2;   // 32 KiB

// dz = p_s ((z_s - z_t) - mu), rounded to bf16, into rows wrow + fn*32 + lane%32 of the tile.
__device__ __forceinline__ void dz_epilogue(const f32x16 (&zs)[4][2], const f32x16 (&zt)[4][2],
                                            const float (&lse2)[2], const float (&mu)[2], __bf16* blk,
                                            int wrow, int v0, int V, bool tail, int lane) {
  const int half = lane >> 5, vlane = v0 + 4 * half, key = (lane >> 1) & 7;
#pragma unroll
  for (int fn = 0; fn < 2; ++fn) {
    __bf16* out = blk + (wrow + fn * 32 + (lane & 31)) * kBK + 4 * half;
#pragma unroll
    for (int fm = 0; fm < 4; ++fm)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float d[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float s = zs[fm][fn][q * 4 + e], t = zt[fm][fn][q * 4 + e];
          d[e] = fast_exp2(fmaf(s, kLog2e, -lse2[fn])) * ((s - t) - mu[fn]);
        }
        if (tail && vlane + fm * 32 + 8 * q >= V) { d[0] = d[1] = d[2] = d[3] = 0.f; }
        uint2 o;
        o.x = pack_bf16(d[0], d[1]);
        o.y = pack_bf16(d[2], d[3]);
        *(uint2*)(out + (fm >> 1) * kSlabBlock + ((((fm & 1) * 4 + q) ^ key) << 3)) = o;
      }
  }
}

// Single-sweep epilogue.  With per-row references fixed in advance (rs2 = m_ref_s*log2e,
// rt2 = m_ref_t*log2e, mu0 ~ E_{p_s}[z_s - z_t]) every exponential is taken relative to the
// same reference in every tile, so the statistics are plain sums,
//   Z_s = sum e_s,  A = sum e_s d,  Z_t = sum e_t,   e_s = exp(z_s - m_ref_s), d = z_s - z_t,
// and two bf16 factors of the unnormalised gradient can be emitted at once, D = d - mu0 and
// E2 = e_s: dz = E2 (D - (mu - mu0)) / Z_s.  mu0 is a per-(row, vocabulary tile) reference
// kept for the combine pass.  D goes to slab rows row0.., E2 to the same rows e2_off elements
// further on.
// B_t = sum e_t z_t (teacher entropy) and cnt = entries ranked above the sampled token are
// only maintained in diagnostics mode.
struct LaneSums { float Z_s[2], A_s[2], Z_t[2], B_t[2]; int cnt[2]; };

template <bool TAIL, bool DIAG, bool WRITE_D, bool WRITE_E2>
__device__ __forceinline__ void single_epilogue(const f32x16 (&zs)[4][2], const f32x16 (&zt)[4][2],
                                                LaneSums& sm, const float (&rs2)[2],
                                                const float (&rt2)[2], float (&mu0)[2],
                                                const float (&zyt)[2], const int (&yid)[2],
                                                __bf16* blk, int64_t e2_off, int wrow,
                                                int v0, int V, int lane, float* mu0_out) {
  const int half = lane >> 5, vlane = v0 + 4 * half, key = (lane >> 1) & 7;
#pragma unroll
  for (int fn = 0; fn < 2; ++fn) {
    __bf16* out = blk + (wrow + fn * 32 + (lane & 31)) * kBK + 4 * half;
    float Zs = sm.Z_s[fn], As = sm.A_s[fn], Zt = sm.Z_t[fn], Bt = sm.B_t[fn];
    int cnt = sm.cnt[fn];
    const int vy = yid[fn] - vlane;        // position of the sampled token among this lane's entries
#pragma unroll
    for (int fm = 0; fm < 4; ++fm)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float e2[4];
        const bool ok = !TAIL || (vlane + fm * 32 + 8 * q) < V;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float s = zs[fm][fn][q * 4 + e], t = zt[fm][fn][q * 4 + e];
          float es = fast_exp2(fmaf(s, kLog2e, -rs2[fn]));
          float et = fast_exp2(fmaf(t, kLog2e, -rt2[fn]));
          float d = s - t;
          if (TAIL && !ok) { es = 0.f; et = 0.f; d = 0.f; }
          Zs += es;
          As = fmaf(es, d, As);
          Zt += et;
          if (DIAG) {
            Bt = fmaf(et, t, Bt);
            cnt += (t > zyt[fn] && (fm * 32 + 8 * q + e) != vy && ok) ? 1 : 0;
          }
          e2[e] = es;
        }
        uint2 o2;
        o2.x = pack_bf16(e2[0], e2[1]); o2.y = pack_bf16(e2[2], e2[3]);
        const int at = (fm >> 1) * kSlabBlock + ((((fm & 1) * 4 + q) ^ key) << 3);
        if (WRITE_E2) *(uint2*)(out + e2_off + at) = o2;
      }
    sm.Z_s[fn] = Zs; sm.A_s[fn] = As; sm.Z_t[fn] = Zt;
    if (DIAG) { sm.B_t[fn] = Bt; sm.cnt[fn] = cnt; }
    if (WRITE_D) {
      // Second factor: D = d - mu0 with mu0 the strip's running mean of d = z_s - z_t under the
      // student weights, this tile included (both half-columns of the row).  A heavy entry
      // dominates the mean of its own tile, so its D is stored small and the correction
      // (mu - mu0) carries its gradient: the rounding of both factors stays proportional to
      // p_s |d - mu| even when the row is peaked and the first vocabulary entries say nothing
      // about mu.  The masked entries of a tail tile have E2 = 0; their D is immaterial.
      const float Zr = Zs + __shfl_xor(Zs, 32, 64), Ar = As + __shfl_xor(As, 32, 64);
      if (Zr > 0.f) mu0[fn] = Ar / Zr;
      const float m0 = mu0[fn];
      if (mu0_out && lane < 32) mu0_out[fn * 32 + lane] = m0;
#pragma unroll
      for (int fm = 0; fm < 4; ++fm)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float dd[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) dd[e] = (zs[fm][fn][q * 4 + e] - m0) - zt[fm][fn][q * 4 + e];
          uint2 o1;
          o1.x = pack_bf16(dd[0], dd[1]); o1.y = pack_bf16(dd[2], dd[3]);
          const int at = (fm >> 1) * kSlabBlock + ((((fm & 1) * 4 + q) ^ key) << 3);
          *(uint2*)(out + at) = o1;
        }
    }
  }
}

template <bool DIAG>
__device__ __forceinline__ void write_sums(LaneSums& sm, float* part, int strips, int strip,
                                           int64_t n_pad, int64_t row0, int lane) {
#pragma unroll
  for (int fn = 0; fn < 2; ++fn) {
    const float Zs = sm.Z_s[fn] + __shfl_xor(sm.Z_s[fn], 32, 64);
    const float As = sm.A_s[fn] + __shfl_xor(sm.A_s[fn], 32, 64);
    const float Zt = sm.Z_t[fn] + __shfl_xor(sm.Z_t[fn], 32, 64);
    const float Bt = DIAG ? sm.B_t[fn] + __shfl_xor(sm.B_t[fn], 32, 64) : 0.f;
    const int cnt = DIAG ? sm.cnt[fn] + __shfl_xor(sm.cnt[fn], 32, 64) : 0;
    if (lane < 32) {
      const int64_t plane = (int64_t)strips * n_pad;
      float* o = part + (int64_t)strip * n_pad + row0 + fn * 32 + lane;
      o[0 * plane] = Zs;
      o[1 * plane] = As;
      o[2 * plane] = Zt;
      if (DIAG) {
        o[3 * plane] = Bt;
        o[4 * plane] = (float)cnt;     // at most V < 2^24: exact
      }
    }
  }
}

// Merge the two half-columns held by lanes l and l^32 and write one strip's partials.
__device__ __forceinline__ void write_partials(LaneStats& st, float* part, int strips, int strip,
                                               int64_t n_pad, int64_t row0, int lane) {
#pragma unroll
  for (int fn = 0; fn < 2; ++fn) {
    merge_mza(st.m_s[fn], st.Z_s[fn], st.A_s[fn], __shfl_xor(st.m_s[fn], 32, 64),
              __shfl_xor(st.Z_s[fn], 32, 64), __shfl_xor(st.A_s[fn], 32, 64));
    merge_mz(st.m_t[fn], st.Z_t[fn], __shfl_xor(st.m_t[fn], 32, 64), __shfl_xor(st.Z_t[fn], 32, 64));
    if (lane < 32) {
      const int64_t plane = (int64_t)strips * n_pad;
      float* o = part + (int64_t)strip * n_pad + row0 + fn * 32 + lane;
      o[0 * plane] = st.m_s[fn];
      o[1 * plane] = st.Z_s[fn];
      o[2 * plane] = st.A_s[fn];
      o[3 * plane] = st.m_t[fn];
      o[4 * plane] = st.Z_t[fn];
    }
  }
}

constexpr int kLogitStage = (kTileVocab + kTileTokens) * kRowBytes;   // 48 KiB
constexpr int kLogitLds = 2 * kLogitStage;

template <bool PASS2>
__global__ __launch_bounds__(256) void logit_pass_kernel(LogitPassArgs a) {
  extern __shared__ __align__(16) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // virtual id -> (group of 4 token tiles, strip, tile in group)
  const int vid = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int per_group = a.tg * a.strips;
  const int tg = vid / per_group, within = vid % per_group;
  const int strip = within / a.tg, tt_local = tg * a.tg + (within % a.tg);
  if (tt_local >= a.n_tiles) return;
  const int tt = a.tile0 + tt_local;
  const int vt_begin = (int)((int64_t)a.vt_total * strip / a.strips);
  const int vt_end = (int)((int64_t)a.vt_total * (strip + 1) / a.strips);

  // token-row stagers (rows fixed for the whole vocabulary walk)
  RowStager<kTileTokens> hs, ht;
  RowStager<kTileVocab> ws, wt;
  {
    const int r = tid >> 3, c = tid & 7;
#pragma unroll
    for (int i = 0; i < kTileTokens / 32; ++i) {
      const int64_t row = a.row_idx[(int64_t)tt * kTileTokens + r + 32 * i];
      hs.p[i] = (const uint4*)(a.h_s + row * a.H_s) + c;
      ht.p[i] = (const uint4*)(a.h_t + row * a.H_t) + c;
    }
  }
  const int waveB = wave * 64 * kRowBytes;   // this wave's 64 token rows in the B tile

  LaneStats st;
  float lse2[2], mu[2];
#pragma unroll
  for (int fn = 0; fn < 2; ++fn) {
    st.m_s[fn] = kNegBig; st.Z_s[fn] = 0.f; st.A_s[fn] = 0.f; st.m_t[fn] = kNegBig; st.Z_t[fn] = 0.f;
    lse2[fn] = 0.f; mu[fn] = 0.f;
    if (PASS2) {
      const int64_t r = (int64_t)tt * kTileTokens + wave * 64 + fn * 32 + (lane & 31);
      lse2[fn] = a.lse2[r];
      mu[fn] = a.mu[r];
    }
  }

  for (int vt = vt_begin; vt < vt_end; ++vt) {
    const int v0 = vt * kTileVocab;
    {
      const int r = tid >> 3, c = tid & 7;
#pragma unroll
      for (int i = 0; i < kTileVocab / 32; ++i) {
        int v = v0 + r + 32 * i;
        v = v < a.V ? v : a.V - 1;               // tail rows: load a valid row, masked below
        ws.p[i] = (const uint4*)(a.W_s + (int64_t)v * a.H_s) + c;
        wt.p[i] = (const uint4*)(a.W_t + (int64_t)v * a.H_t) + c;
      }
    }
    f32x16 zt[4][2], zs[4][2];
#pragma unroll
    for (int fm = 0; fm < 4; ++fm)
#pragma unroll
      for (int fn = 0; fn < 2; ++fn)
#pragma unroll
        for (int e = 0; e < 16; ++e) { zt[fm][fn][e] = 0.f; zs[fm][fn][e] = 0.f; }
    gemm_kloop<kTileVocab, kTileTokens, 4, 2>(zt, wt, ht, 0, a.H_t / kBK, lds, kLogitStage, 0, waveB, tid);
    gemm_kloop<kTileVocab, kTileTokens, 4, 2>(zs, ws, hs, 0, a.H_s / kBK, lds, kLogitStage, 0, waveB, tid);

    const bool tail = v0 + kTileVocab > a.V;
    if (!PASS2) stats_epilogue(zs, zt, st, v0, a.V, tail, lane);
    else dz_epilogue(zs, zt, lse2, mu, a.slab + ((int64_t)tt_local * (a.Vp / kBK) + 2 * vt) * kSlabBlock,
                     wave * 64, v0, a.V, tail, lane);
  }
  if (!PASS2)
    write_partials(st, a.part, a.strips, strip, a.n_pad, (int64_t)tt * kTileTokens + wave * 64, lane);
}

// ---------------------------------------------------------------------------------------
// Logit passes, direct global->LDS staging.
//
// Same tile, MFMA roles and epilogues as logit_pass_kernel, but the k-tiles are moved by
// global_load_lds_dwordx4 (no register staging) into a three-stage LDS ring, two k-steps
// ahead of the MFMAs.  One wave instruction moves 8 rows x 128 B: lane l lands at
// base + 16 l, i.e. row l/8, chunk position l%8, and therefore fetches global chunk
// (l%8) ^ swizzle(row).  The teacher and student k-loops form one pipeline of
// H_t/64 + H_s/64 steps per vocabulary tile.
//
// The loads are written as inline assembly (M0 = LDS destination of the wave, scalar base
// + 32-bit lane offset) and waited for with explicit s_waitcnt vmcnt(N): the loads return
// in order, so "at most the 12 loads of the next stage outstanding" means this stage has
// landed.  Compiler-issued loads in between only make the count larger, i.e. the wait
// longer.  Requires rows * H * 2 bytes < 4 GiB per operand (32-bit lane offsets).
// ---------------------------------------------------------------------------------------
constexpr int kDmaStages = 3;
constexpr int kDmaLds = kDmaStages * kLogitStage;           // 144 KiB
constexpr int kDmaPerWave = (kTileVocab + kTileTokens) / 8 / 4;   // 12 wave-loads per stage

__device__ __forceinline__ void dma16(uint32_t lds_dst, uint32_t voff, const char* sbase) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_dst), "v"(voff), "s"(sbase) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// Row images.  The direct-to-LDS logit kernel reads all four operands as LDS images of its
// k-steps: [rows, H] row-major (optionally gathered through row_idx) is re-laid as tiles of
// `th` consecutive rows; block (tile, kt) holds their k-entries 64 kt .. 64 kt + 63, row r at
// r * 128 B, its 16-byte chunk c at chunk position c ^ ((r >> 1) & 7); rows >= n_rows are
// zero.  Blocks of one tile are consecutive in kt.  Every wave-load then moves 1 KiB of
// consecutive bytes and no operand needs 32-bit lane offsets from its base.
struct RowImageArgs {
  const uint4* src; uint4* img; const int32_t* row_idx;
  int64_t n_rows; int H, nk, th;
};

__global__ __launch_bounds__(256) void row_image_kernel(RowImageArgs a) {
  const int kt = blockIdx.x;
  const int64_t tile = blockIdx.y;
  uint4* blk = a.img + ((tile * a.nk + kt) * a.th) * 8;
  for (int q = threadIdx.x; q < a.th * 8; q += 256) {
    const int r = q >> 3, pos = q & 7, c = pos ^ ((r >> 1) & 7);
    const int64_t row = tile * a.th + r;
    uint4 v = {0u, 0u, 0u, 0u};
    if (row < a.n_rows) {
      const int64_t src_row = a.row_idx ? (int64_t)a.row_idx[row] : row;
      v = a.src[src_row * (a.H >> 3) + kt * 8 + c];
    }
    blk[q] = v;
  }
}

constexpr int kImgABytes = kTileVocab * kRowBytes;    // 16 KiB: one W block
constexpr int kImgBBytes = kTileTokens * kRowBytes;   // 32 KiB: one h block

// Wave-load I (0..11) of this wave for one stage: KiB (wave + 4 I) of the A block, then of
// the B block; lane l moves bytes 16 l .. 16 l + 15 of that KiB.
template <int I>
__device__ __forceinline__ void dma_one(uint32_t lds_stage, int wave, uint32_t voff, const char* sA,
                                        const char* sB) {
  if constexpr (I < kTileVocab / 32)
    dma16(lds_stage + (uint32_t)(wave + 4 * I) * 1024u, voff, sA + (wave + 4 * I) * 1024);
  else
    dma16(lds_stage + (uint32_t)(kTileVocab / 8 + wave + 4 * (I - kTileVocab / 32)) * 1024u, voff,
          sB + (wave + 4 * (I - kTileVocab / 32)) * 1024);
}

// One staged k-step (4 sub-steps of 8 MFMAs) of the 128 x 64 wave tile.  On entry fa[0],
// fb[0] hold the fragments of sub-step 0.  The instruction order is pinned: after each MFMA
// one or two side operations are issued in its shadow -- an LDS read of a fragment of the
// next sub-step (fragments are double-buffered) and, when ISSUE, one of the 12 global->LDS
// loads of the stage two k-steps ahead -- so that neither the LDS latency nor the
// vector-memory issue holds up the matrix pipe.  The one barrier of the k-step sits before
// the last sub-step: by then every fragment of this stage is in registers, and the last
// sub-step's MFMAs cover the reads of the next stage's first fragments (stage `nxt`, whose
// loads were issued one k-step earlier and are waited for here).  LAST: no next stage in
// this vocabulary tile; no barrier and no fragment reads.
template <bool ISSUE, bool LAST>
__device__ __forceinline__ void sweep_kstep(f32x16 (&acc)[4][2], bf16x8 (&fa)[2][4], bf16x8 (&fb)[2][2],
                                            const char* curA, const char* curB, const char* nxtA,
                                            const char* nxtB, int lane, uint32_t lds_stage, int wave,
                                            uint32_t voff, const char* sA, const char* sB) {
  const int key = (lane >> 1) & 7, half = lane >> 5;
  const int rowoff = (lane & 31) * kRowBytes;
  int sw[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) sw[kk] = rowoff + (((kk * 2 + half) ^ key) << 4);
#define ADWIN_FENCE __builtin_amdgcn_sched_barrier(0);
#define ADWIN_RA(TA, KK, I) fa[((KK) + 1) & 1][I] = *(const bf16x8*)((TA) + (I) * 32 * kRowBytes + sw[((KK) + 1) & 3]); ADWIN_FENCE
#define ADWIN_RB(TB, KK, I) fb[((KK) + 1) & 1][I] = *(const bf16x8*)((TB) + (I) * 32 * kRowBytes + sw[((KK) + 1) & 3]); ADWIN_FENCE
#define ADWIN_MM(KK, FMI, FNI)                                                                  \
  acc[FMI][FNI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[(KK) & 1][FMI], fb[(KK) & 1][FNI], \
                                                          acc[FMI][FNI], 0, 0, 0);              \
  ADWIN_FENCE
#define ADWIN_DMA(I) if constexpr (ISSUE) { dma_one<I>(lds_stage, wave, voff, sA, sB); ADWIN_FENCE }
  // sub-step KK: 8 MFMAs; reads of the next sub-step's fragments from (TA, TB) when READ
#define ADWIN_SUB(KK, READ, TA, TB, D0, D1, D2)                         \
  ADWIN_MM(KK, 0, 0) if constexpr (READ) { ADWIN_RA(TA, KK, 0) }        \
  ADWIN_MM(KK, 0, 1) if constexpr (READ) { ADWIN_RB(TB, KK, 0) }        \
  ADWIN_MM(KK, 1, 0) if constexpr (READ) { ADWIN_RA(TA, KK, 1) }        \
  ADWIN_MM(KK, 1, 1) if constexpr (READ) { ADWIN_RB(TB, KK, 1) }        \
  ADWIN_MM(KK, 2, 0) if constexpr (READ) { ADWIN_RA(TA, KK, 2) }        \
  ADWIN_MM(KK, 2, 1) if constexpr (READ) { ADWIN_RA(TA, KK, 3) } ADWIN_DMA(D0) \
  ADWIN_MM(KK, 3, 0) ADWIN_DMA(D1)                                      \
  ADWIN_MM(KK, 3, 1) ADWIN_DMA(D2)
  ADWIN_FENCE
  ADWIN_SUB(0, true, curA, curB, 0, 1, 2)
  ADWIN_SUB(1, true, curA, curB, 3, 4, 5)
  ADWIN_SUB(2, true, curA, curB, 6, 7, 8)
  if constexpr (!LAST) {
    // loads issued after those of the next stage: the 9 above (none when !ISSUE)
    if constexpr (ISSUE) asm volatile("s_waitcnt vmcnt(9) lgkmcnt(0)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __syncthreads();
  }
  ADWIN_FENCE
  ADWIN_SUB(3, !LAST, nxtA, nxtB, 9, 10, 11)
#undef ADWIN_SUB
#undef ADWIN_DMA
#undef ADWIN_MM
#undef ADWIN_RB
#undef ADWIN_RA
#undef ADWIN_FENCE
}

template <int MODE>
__global__ __launch_bounds__(256) void logit_pass_dma_kernel(LogitPassArgs a) {
  extern __shared__ __align__(16) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int vid = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int per_group = a.tg * a.strips;
  const int tg = vid / per_group, within = vid % per_group;
  const int strip = within / a.tg, tt_local = tg * a.tg + (within % a.tg);
  if (tt_local >= a.n_tiles) return;
  const int tt = a.tile0 + tt_local;
  const int vt_begin = (int)((int64_t)a.vt_total * strip / a.strips);
  const int vt_end = (int)((int64_t)a.vt_total * (strip + 1) / a.strips);
  if (vt_begin >= vt_end) return;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;

  const uint32_t voff = (uint32_t)lane * 16u;
  const int waveA = 0, waveB = kTileVocab * kRowBytes + wave * 64 * kRowBytes;
  const int nk_t = a.H_t / kBK, nk_s = a.H_s / kBK, nk = nk_t + nk_s;   // each >= 2 on this path
  // blocks of this token tile (fixed) and of vocabulary tile vt, teacher and student
  const char* sHt = a.ht_img + (int64_t)tt * nk_t * kImgBBytes;
  const char* sHs = a.hs_img + (int64_t)tt * nk_s * kImgBBytes;
  auto blocks_wt = [&](int vt) { return a.Wt_img + (int64_t)vt * nk_t * kImgABytes; };
  auto blocks_ws = [&](int vt) { return a.Ws_img + (int64_t)vt * nk_s * kImgABytes; };

  LaneStats st;
  LaneSums sm;
  constexpr bool kDiag = MODE == kModeSingleDiag || MODE == kModeSingleE2Diag || MODE == kModeSingleFwdDiag;
  constexpr bool kWriteE2 = MODE < kModeSingleFwd;
  constexpr bool kWriteD = MODE == kModeSingle || MODE == kModeSingleDiag;
  constexpr bool kSingle = MODE >= kModeSingle;
  float lse2[2], mu[2], rs2[2], rt2[2];   // per-row inputs of the dz / single-sweep epilogues
  float zyt[2];
  int yid[2];
#pragma unroll
  for (int fn = 0; fn < 2; ++fn) {
    st.m_s[fn] = kNegBig; st.Z_s[fn] = 0.f; st.A_s[fn] = 0.f; st.m_t[fn] = kNegBig; st.Z_t[fn] = 0.f;
    sm.Z_s[fn] = 0.f; sm.A_s[fn] = 0.f; sm.Z_t[fn] = 0.f; sm.B_t[fn] = 0.f; sm.cnt[fn] = 0;
    lse2[fn] = 0.f; mu[fn] = 0.f; rs2[fn] = 0.f; rt2[fn] = 0.f; zyt[fn] = 0.f; yid[fn] = -1;
    const int64_t r = (int64_t)tt * kTileTokens + wave * 64 + fn * 32 + (lane & 31);
    if (MODE == kModeDz) {
      lse2[fn] = a.lse2[r];
      mu[fn] = a.mu[r];
    } else if (kSingle) {
      rs2[fn] = a.ref_s2[r];
      rt2[fn] = a.ref_t2[r];
      mu[fn] = a.mu0[r];
      if (kDiag) { zyt[fn] = a.zy_t[r]; yid[fn] = a.yid[r]; }
    }
  }

  // The k-steps of all vocabulary tiles of the strip form one pipeline: per tile nk_t
  // teacher steps, then nk_s student steps; step g is staged into ring slot g % 3 two steps
  // before it is consumed, also across the tile boundary (the next tile's first two steps
  // are loaded during this tile's last two, i.e. before and under the epilogue).
  uint32_t wr = 0, rd = 0;     // ring slots of the next step to load / to consume
  auto slot_inc = [](uint32_t x) { return x + 1 == kDmaStages ? 0u : x + 1; };
  {
    const char* sWt = blocks_wt(vt_begin);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint32_t dst = lds0 + wr * kLogitStage;
      const char* sA = sWt + i * kImgABytes;
      const char* sB = sHt + i * kImgBBytes;
      dma_one<0>(dst, wave, voff, sA, sB); dma_one<1>(dst, wave, voff, sA, sB);
      dma_one<2>(dst, wave, voff, sA, sB); dma_one<3>(dst, wave, voff, sA, sB);
      dma_one<4>(dst, wave, voff, sA, sB); dma_one<5>(dst, wave, voff, sA, sB);
      dma_one<6>(dst, wave, voff, sA, sB); dma_one<7>(dst, wave, voff, sA, sB);
      dma_one<8>(dst, wave, voff, sA, sB); dma_one<9>(dst, wave, voff, sA, sB);
      dma_one<10>(dst, wave, voff, sA, sB); dma_one<11>(dst, wave, voff, sA, sB);
      wr = slot_inc(wr);
    }
  }
  for (int vt = vt_begin; vt < vt_end; ++vt) {
    const int v0 = vt * kTileVocab;
    const char* sWt = blocks_wt(vt);
    const char* sWs = blocks_ws(vt);
    f32x16 zt[4][2], zs[4][2];
#pragma unroll
    for (int fm = 0; fm < 4; ++fm)
#pragma unroll
      for (int fn = 0; fn < 2; ++fn)
#pragma unroll
        for (int e = 0; e < 16; ++e) { zt[fm][fn][e] = 0.f; zs[fm][fn][e] = 0.f; }

    // step 0 of this tile has landed once at most the 12 loads of step 1 are outstanding
    wait_vm<kDmaPerWave>();
    __syncthreads();
    bf16x8 fa[2][4], fb[2][2];
    {
      const char* cur = lds + rd * kLogitStage;
      const int key = (lane >> 1) & 7, half = lane >> 5;
      const int sw0 = (lane & 31) * kRowBytes + ((half ^ key) << 4);
#pragma unroll
      for (int i = 0; i < 4; ++i) fa[0][i] = *(const bf16x8*)(cur + waveA + i * 32 * kRowBytes + sw0);
#pragma unroll
      for (int i = 0; i < 2; ++i) fb[0][i] = *(const bf16x8*)(cur + waveB + i * 32 * kRowBytes + sw0);
    }
    // one k-step: consume slot rd, prefetch fragments from the following slot, load into wr
    auto step = [&](auto issue_c, auto last_c, f32x16 (&acc)[4][2], const char* sA, const char* sB) {
      constexpr bool kIssue = decltype(issue_c)::value, kLast = decltype(last_c)::value;
      const char* cur = lds + rd * kLogitStage;
      const uint32_t rn = slot_inc(rd);
      const char* nxt = lds + rn * kLogitStage;
      sweep_kstep<kIssue, kLast>(acc, fa, fb, cur + waveA, cur + waveB, nxt + waveA, nxt + waveB, lane,
                                 lds0 + wr * kLogitStage, wave, voff, sA, sB);
      if (kIssue) wr = slot_inc(wr);
      rd = rn;
    };
    const std::true_type yes{};
    const std::false_type no{};
    int s = 0;
    for (; s + 2 < nk_t; ++s)                  // teacher k-steps loading teacher k-steps
      step(yes, no, zt, sWt + (s + 2) * kImgABytes, sHt + (s + 2) * kImgBBytes);
    for (; s < nk_t; ++s) {                    // last two teacher k-steps load student k-steps 0, 1
      const int n = s + 2 - nk_t;
      step(yes, no, zt, sWs + n * kImgABytes, sHs + n * kImgBBytes);
    }
    for (; s + 2 < nk; ++s) {                  // student k-steps loading student k-steps
      const int n = s + 2 - nk_t;
      step(yes, no, zs, sWs + n * kImgABytes, sHs + n * kImgBBytes);
    }
    if (vt + 1 < vt_end) {                     // last two: load the next tile's teacher k-steps 0, 1
      const char* sWn = blocks_wt(vt + 1);
      step(yes, no, zs, sWn, sHt);
      step(yes, yes, zs, sWn + kImgABytes, sHt + kImgBBytes);
    } else {
      step(no, no, zs, sWs, sHs);
      step(no, yes, zs, sWs, sHs);
    }
    const bool tail = v0 + kTileVocab > a.V;
    if (MODE == kModeStats) {
      stats_epilogue(zs, zt, st, v0, a.V, tail, lane);
    } else {
      __bf16* blk = a.slab + ((int64_t)tt_local * (a.Vp / kBK) + 2 * vt) * kSlabBlock;
      float* m0t = a.mu0t ? a.mu0t + (int64_t)vt * a.mu0t_stride + (int64_t)tt_local * kTileTokens + wave * 64
                          : nullptr;
      if (MODE == kModeDz) {
        dz_epilogue(zs, zt, lse2, mu, blk, wave * 64, v0, a.V, tail, lane);
      } else if (tail) {
        single_epilogue<true, kDiag, kWriteD, kWriteE2>(zs, zt, sm, rs2, rt2, mu, zyt, yid, blk, a.e2_off, wave * 64, v0, a.V, lane, m0t);
      } else {
        single_epilogue<false, kDiag, kWriteD, kWriteE2>(zs, zt, sm, rs2, rt2, mu, zyt, yid, blk, a.e2_off, wave * 64, v0, a.V, lane, m0t);
      }
    }
  }
  const int64_t row0 = (int64_t)tt * kTileTokens + wave * 64;
  if (MODE == kModeStats) write_partials(st, a.part, a.strips, strip, a.n_pad, row0, lane);
  else if (kSingle) write_sums<kDiag>(sm, a.part, a.strips, strip, a.n_pad, row0, lane);
}

// ---------------------------------------------------------------------------------------
// Merge of the strip partials, KL_t and c_t.  One wave per computed row.
// ---------------------------------------------------------------------------------------
struct MergeArgs {
  const float* part; int strips; int64_t n_pad; int64_t n_rows;
  const int32_t* row_idx;
  const __bf16* h_s; const __bf16* h_t; const __bf16* W_s; const __bf16* W_t;
  int H_s, H_t, V;
  const int32_t* ids;
  float* lse2; float* mu; float* klr;
  float* kl; float* c;
  uint32_t* status;
  // teacher-side diagnostics (single-sweep merge only); part planes 3 and 4 hold
  // sum e_t z_t and the rank count when `diag` is set
  int diag;
  float* t_logp; float* t_entropy; int32_t* t_rank;
  float* cr;     // [n_pad] c_t per computed row, for the sampled estimator (else NULL)
};

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

__global__ __launch_bounds__(256) void merge_stats_kernel(MergeArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= a.n_pad) return;
  const int64_t plane = (int64_t)a.strips * a.n_pad;
  float ms = kNegBig, Zs = 0.f, A = 0.f, mt = kNegBig, Zt = 0.f;
  if (lane < a.strips) {
    const float* p = a.part + (int64_t)lane * a.n_pad + r;
    ms = p[0]; Zs = p[plane]; A = p[2 * plane]; mt = p[3 * plane]; Zt = p[4 * plane];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    merge_mza(ms, Zs, A, __shfl_xor(ms, o, 64), __shfl_xor(Zs, o, 64), __shfl_xor(A, o, 64));
    merge_mz(mt, Zt, __shfl_xor(mt, o, 64), __shfl_xor(Zt, o, 64));
  }
  const float lse_s = ms + logf(Zs), lse_t = mt + logf(Zt);
  const float mu = A / Zs;                  // E_{p_s}[z_s - z_t]
  const float kl = kl_from_sums(mu, ms - mt, Zs, Zt);
  if (lane == 0) {
    a.lse2[r] = lse_s * kLog2e;
    a.mu[r] = mu;
    a.klr[r] = kl;
  }
  if (r >= a.n_rows) return;                // padding rows feed pass 2 only
  const int64_t t = a.row_idx[r];
  float c = 0.f;
  uint32_t flag = 0;
  if (a.ids && a.c) {
    const int y = a.ids[t];
    if (y >= 0 && y < a.V) {
      const float zy_s = dot_bf16_row(a.h_s + t * a.H_s, a.W_s + (int64_t)y * a.H_s, a.H_s, lane);
      const float zy_t = dot_bf16_row(a.h_t + t * a.H_t, a.W_t + (int64_t)y * a.H_t, a.H_t, lane);
      c = (zy_s - lse_s) - (zy_t - lse_t);
    } else {
      flag |= ADWIN_DEV_BAD_ID;
    }
  }
  if (!(fabsf(lse_s) < 3.0e38f) || !(fabsf(lse_t) < 3.0e38f) || !(fabsf(kl) < 3.0e38f))
    flag |= ADWIN_DEV_NONFINITE;
  if (lane == 0) {
    if (flag && a.status) atomicOr(a.status, flag);
    if (a.kl) a.kl[t] = kl;
    if (a.c) a.c[t] = c;
  }
}

// ---------------------------------------------------------------------------------------
// Single-sweep mode: per-row references from the online statistics of vocabulary tile 0,
// and the merge of the fixed-reference strip sums.
// ---------------------------------------------------------------------------------------
__global__ void make_refs_kernel(const float* __restrict__ part /* [5][1][n_pad] */, int64_t n_pad,
                                 const float* __restrict__ zy_s, const float* __restrict__ zy_t,
                                 const int32_t* __restrict__ yid, float* ref_s2, float* ref_t2,
                                 float* mu0) {
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_pad) return;
  float ms = part[r], Zs = part[n_pad + r], A = part[2 * n_pad + r], mt = part[3 * n_pad + r];
  if (yid && yid[r] >= 0) {
    // The sampled token joins the first vocabulary tile as a sample of the row: drawn from the
    // student, it sits where the mass is, which the first 128 entries of a peaked row do not.
    // The references rise to its logits (the exponentials of the sweep stay near 1 at the
    // row maximum instead of growing with the gap to the first tile), and mu0 becomes the
    // self-normalised estimate of E_p[z_s - z_t] over the tile's entries and the token.
    const float zs = zy_s[r], zt = zy_t[r];
    const float rs = fmaxf(ms, zs);
    const float sc = fast_exp2((ms - rs) * kLog2e);
    Zs *= sc; A *= sc;
    if (yid[r] >= kTileVocab) {           // not already one of the tile's entries
      const float ey = fast_exp2((zs - rs) * kLog2e);
      Zs += ey;
      A = fmaf(ey, zs - zt, A);
    }
    ms = rs;
    mt = fmaxf(mt, zt);
  }
  ref_s2[r] = ms * kLog2e;
  ref_t2[r] = mt * kLog2e;
  mu0[r] = A / Zs;
}

struct MergeSingleArgs {
  MergeArgs m;                 // part: [3][strips][n_pad] sums Z_s, A, Z_t
  const float* ref_s2; const float* ref_t2;
  float* mu_out; float* inv_z;
  int64_t row0, rows;          // computed rows [row0, row0 + rows) of this launch (one slab)
};

__global__ __launch_bounds__(256) void merge_single_kernel(MergeSingleArgs b) {
  const MergeArgs& a = b.m;
  const int lane = threadIdx.x & 63;
  const int64_t r = b.row0 + (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= b.row0 + b.rows) return;
  const int64_t plane = (int64_t)a.strips * a.n_pad;
  float Zs = 0.f, A = 0.f, Zt = 0.f, Bt = 0.f, cnt = 0.f;
  if (lane < a.strips) {
    const float* p = a.part + (int64_t)lane * a.n_pad + r;
    Zs = p[0]; A = p[plane]; Zt = p[2 * plane];
    if (a.diag) { Bt = p[3 * plane]; cnt = p[4 * plane]; }
  }
  Zs = wave_sum(Zs); A = wave_sum(A); Zt = wave_sum(Zt);
  if (a.diag) { Bt = wave_sum(Bt); cnt = wave_sum(cnt); }
  const float lse_s = b.ref_s2[r] * kLn2 + logf(Zs), lse_t = b.ref_t2[r] * kLn2 + logf(Zt);
  const float mu = A / Zs;                  // E_{p_s}[z_s - z_t]
  const float kl = kl_from_sums(mu, (b.ref_s2[r] - b.ref_t2[r]) * kLn2, Zs, Zt);
  if (lane == 0) {
    b.mu_out[r] = mu;
    b.inv_z[r] = 1.f / Zs;
    a.klr[r] = kl;
  }
  if (r >= a.n_rows) return;
  const int64_t t = a.row_idx[r];
  float c = 0.f, logp_t = 0.f;
  bool have_y = false;
  uint32_t flag = 0;
  if (a.ids && (a.c || a.t_logp || a.t_rank || a.cr)) {
    const int y = a.ids[t];
    if (y >= 0 && y < a.V) {
      const float zy_s = dot_bf16_row(a.h_s + t * a.H_s, a.W_s + (int64_t)y * a.H_s, a.H_s, lane);
      const float zy_t = dot_bf16_row(a.h_t + t * a.H_t, a.W_t + (int64_t)y * a.H_t, a.H_t, lane);
      c = (zy_s - lse_s) - (zy_t - lse_t);
      logp_t = zy_t - lse_t;
      have_y = true;
    } else {
      flag |= ADWIN_DEV_BAD_ID;
    }
  }
  if (!(fabsf(lse_s) < 3.0e38f) || !(fabsf(lse_t) < 3.0e38f) || !(fabsf(kl) < 3.0e38f) ||
      !(fabsf(A) < 3.0e38f))
    flag |= ADWIN_DEV_NONFINITE;
  if (lane == 0) {
    if (flag && a.status) atomicOr(a.status, flag);
    if (a.kl) a.kl[t] = kl;
    if (a.c) a.c[t] = c;
    if (a.t_logp) a.t_logp[t] = logp_t;
    // H[p_t] = lse_t - E_{p_t}[z_t]; both sums are relative to the same reference
    if (a.t_entropy) a.t_entropy[t] = lse_t - Bt / Zt;
    if (a.t_rank) a.t_rank[t] = have_y ? (int32_t)cnt + 1 : 0;
    if (a.cr) a.cr[r] = c;
  }
}

// Logits of the sampled token under both models, z_s[y_t] = h_s . W_s[y_t] and
// z_t[y_t] = h_t . W_t[y_t], and the token id (-1 when there is none or it is out of range),
// per computed row.  The references of the single sweep are built from them (make_refs_kernel)
// and the diagnostics sweep compares against z_t[y_t] to count the entries the teacher ranks
// above y_t (Sec. 3.1).  One wave per row.
struct TokenLogitArgs {
  const int32_t* row_idx; const int32_t* ids;
  const __bf16* h_s; const __bf16* W_s; const __bf16* h_t; const __bf16* W_t;
  int H_s, H_t, V;
  int64_t n_pad;
  float* zy_s; float* zy_t; int32_t* yid;
};

__global__ __launch_bounds__(256) void token_logit_kernel(TokenLogitArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= a.n_pad) return;
  const int64_t t = a.row_idx[r];
  const int y = a.ids ? a.ids[t] : -1;
  float zs = 0.f, zt = 0.f;
  const bool ok = y >= 0 && y < a.V;
  if (ok) {
    zs = dot_bf16_row(a.h_s + t * a.H_s, a.W_s + (int64_t)y * a.H_s, a.H_s, lane);
    zt = dot_bf16_row(a.h_t + t * a.H_t, a.W_t + (int64_t)y * a.H_t, a.H_t, lane);
  }
  if (lane == 0) { a.zy_s[r] = zs; a.zy_t[r] = zt; a.yid[r] = ok ? y : -1; }
}

// ---------------------------------------------------------------------------------------
// Tile images.  Both operands of the gradient GEMM live in memory as the exact LDS images
// of its k-steps: block (tile, kt) is 256 rows x 64 k-entries = 32 KiB, row r at r * 128 B,
// its 16-byte chunk c (k-entries 8 c .. 8 c + 7) at chunk position c ^ ((r >> 1) & 7).
// Blocks of one tile are consecutive in kt, so a workgroup streams each operand as one
// sequential run and every wave-load moves 1 KiB of consecutive bytes.
// ---------------------------------------------------------------------------------------
constexpr int kImgElems = kGradTile * kBK;            // bf16 elements per block
constexpr int kImgBytes = kImgElems * 2;              // 32 KiB

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
};

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
    if (r < a.n_rows) {
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
    } else {
      const float dl = a.mu[r] - a.mu0t[(int64_t)(kt >> 1) * a.mu0t_stride + rt * kTileTokens + (q >> 3)];
      const uint4 x = p1[q];
      d[0] = (bf16_lo(x.x) - dl) * (bf16_lo(y.x) * iz); d[1] = (bf16_hi(x.x) - dl) * (bf16_hi(y.x) * iz);
      d[2] = (bf16_lo(x.y) - dl) * (bf16_lo(y.y) * iz); d[3] = (bf16_hi(x.y) - dl) * (bf16_hi(y.y) * iz);
      d[4] = (bf16_lo(x.z) - dl) * (bf16_lo(y.z) * iz); d[5] = (bf16_hi(x.z) - dl) * (bf16_hi(y.z) * iz);
      d[6] = (bf16_lo(x.w) - dl) * (bf16_lo(y.w) * iz); d[7] = (bf16_hi(x.w) - dl) * (bf16_hi(y.w) * iz);
      uint4 o;
      o.x = pack_bf16(d[0], d[1]); o.y = pack_bf16(d[2], d[3]);
      o.z = pack_bf16(d[4], d[5]); o.w = pack_bf16(d[6], d[7]);
      p1[q] = o;
    }
    if (TR) {
#pragma unroll
      for (int e = 0; e < 8; ++e) dz[i][e] = d[e];
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
struct HstImageArgs {
  const uint16_t* h_s; const int32_t* row_idx;
  int64_t row0;
  int H, nkr;
  uint16_t* img;
};

__global__ __launch_bounds__(256) void hst_image_kernel(HstImageArgs a) {
  __shared__ uint16_t tile[kBK][kGradTile + 2];
  const int kr = blockIdx.x, ht = blockIdx.y, tid = threadIdx.x;
  for (int i = 0; i < kBK; ++i) {
    const int64_t r = a.row0 + (int64_t)kr * kBK + i;
    const int h = ht * kGradTile + tid;
    tile[i][tid] = h < a.H ? a.h_s[(int64_t)a.row_idx[r] * a.H + h] : (uint16_t)0;
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
// LDS, three for A and two for B, by direct global->LDS loads.  Per k-step a wave issues
// its 16 wave-loads of the k-step after next in the shadow of MFMAs (see grad_kstep), so
// that they have a k-step or more (upwards of 2000 matrix-pipe cycles) to land.  The one
// barrier per k-step sits before the last of the four k16 sub-steps: by then every fragment
// of the current blocks is in registers, so the last sub-step's MFMAs cover the LDS reads of
// the next blocks' first fragments and the matrix pipe never waits for LDS after a barrier.
// ---------------------------------------------------------------------------------------
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

constexpr int kGradABufs = 3;                                 // A blocks in flight or in use
constexpr int kGradBOff = kGradABufs * kImgBytes;             // the two B buffers follow
constexpr int kGradLds = (kGradABufs + 2) * kImgBytes;        // 160 KiB

// LOADS: in k-step s the A block of k-step s + 2 is loaded in sub-step 1 (into the third A
// buffer, which no wave reads any more once it has passed the previous step's barrier) and
// the B block of k-step s + 2 in sub-step 3, after this step's barrier, into the B buffer
// this step has just finished reading.  The A blocks are the stream that comes from HBM (a
// slab block is used by the h tiles of one row tile and never again) and get a lead of a
// k-step and a half, the B blocks, shared by every row tile and mostly found in the L2, one
// k-step.  Loads return in order: the wait before the barrier leaves the youngest eight,
// this step's A loads, in flight.
template <bool LOADS, bool LAST>
__device__ __forceinline__ void grad_kstep(f32x16 (&acc)[4][4], bf16x8 (&fa)[2][4], bf16x8 (&fb)[2][4],
                                           const char* curA, const char* curB, const char* nxtA,
                                           const char* nxtB, int lane, uint32_t lds_a2, uint32_t lds_b2,
                                           uint32_t voff, const char* sB2, const char* sA2) {
  const int key = (lane >> 1) & 7, half = lane >> 5;
  const int rowoff = (lane & 31) * kRowBytes;
  int sw[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) sw[kk] = rowoff + (((kk * 2 + half) ^ key) << 4);
#define ADWIN_FENCE __builtin_amdgcn_sched_barrier(0);
#define ADWIN_MM(KK, I, J)                                                                    \
  acc[I][J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[(KK) & 1][I], fb[(KK) & 1][J],       \
                                                      acc[I][J], 0, 0, 0);                    \
  ADWIN_FENCE
  // side operation M (0..15) in the shadow of MFMA M of sub-step KK: fragment reads of the
  // next sub-step, then (sub-steps 1 and 3) the wave-loads of the k-step after next: 4 KiB
  // groups d = 0..7 of the A block, then of the B block, each offset by this wave's 1 KiB
#define ADWIN_SIDE(KK, M)                                                                           \
  if constexpr ((KK) < 3 && (M) < 8) {                                                              \
    if constexpr (((M) & 1) == 0)                                                                   \
      fa[((KK) + 1) & 1][((M) >> 1) & 3] = *(const bf16x8*)(curA + (((M) >> 1) & 3) * 32 * kRowBytes + sw[(KK) + 1]); \
    else                                                                                            \
      fb[((KK) + 1) & 1][((M) >> 1) & 3] = *(const bf16x8*)(curB + (((M) >> 1) & 3) * 32 * kRowBytes + sw[(KK) + 1]); \
    ADWIN_FENCE                                                                                     \
  } else if constexpr ((KK) == 1 && (M) >= 8 && LOADS) {                                            \
    dma16(lds_a2 + (uint32_t)((M) - 8) * 4096u, voff, sA2 + ((M) - 8) * 4096);                      \
    ADWIN_FENCE                                                                                     \
  } else if constexpr ((KK) == 3 && (M) >= 8 && LOADS) {                                            \
    dma16(lds_b2 + (uint32_t)((M) - 8) * 4096u, voff, sB2 + ((M) - 8) * 4096);                      \
    ADWIN_FENCE                                                                                     \
  } else if constexpr ((KK) == 3 && (M) < 8 && !LAST) {                                             \
    if constexpr (((M) & 1) == 0)                                                                   \
      fa[0][((M) >> 1) & 3] = *(const bf16x8*)(nxtA + (((M) >> 1) & 3) * 32 * kRowBytes + sw[0]);               \
    else                                                                                            \
      fb[0][((M) >> 1) & 3] = *(const bf16x8*)(nxtB + (((M) >> 1) & 3) * 32 * kRowBytes + sw[0]);               \
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
#undef ADWIN_SUB
#undef ADWIN_ROW
#undef ADWIN_SIDE
#undef ADWIN_MM
#undef ADWIN_FENCE
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
  const uint32_t voff = (uint32_t)lane * 16u;
  const char* sA = (const char*)a.slab + ((int64_t)rt * a.nk_total + k_begin) * kImgBytes + wave * 1024;
  const char* sB = (const char*)a.WsT + ((int64_t)ht * a.nk_total + k_begin) * kImgBytes + wave * 1024;
  const uint32_t ldsw = lds0 + (uint32_t)wave * 1024u;

  f32x16 acc[4][4];
#pragma unroll
  for (int fm = 0; fm < 4; ++fm)
#pragma unroll
    for (int fn = 0; fn < 4; ++fn)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[fm][fn][e] = 0.f;

  if (nk > 0) {
    // blocks of the first k-step, then its first fragments
#pragma unroll
    for (int d = 0; d < 8; ++d) {
      dma16(ldsw + (uint32_t)d * 4096u, voff, sA + d * 4096);
      dma16(ldsw + (uint32_t)kGradBOff + (uint32_t)d * 4096u, voff, sB + d * 4096);
    }
    wait_vm<0>();
    __syncthreads();
    bf16x8 fa[2][4], fb[2][4];
    const int waveA = wm * 128 * kRowBytes, waveB = kGradBOff + wn * 128 * kRowBytes;
    {
      const int key = (lane >> 1) & 7, half = lane >> 5;
      const int sw0 = (lane & 31) * kRowBytes + ((half ^ key) << 4);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        fa[0][i] = *(const bf16x8*)(lds + waveA + i * 32 * kRowBytes + sw0);
        fb[0][i] = *(const bf16x8*)(lds + waveB + i * 32 * kRowBytes + sw0);
      }
    }
    // blocks of k-step 1 (k-step s of the loop loads those of k-step s + 2)
    if (nk > 1) {
#pragma unroll
      for (int d = 0; d < 8; ++d) dma16(ldsw + kImgBytes + (uint32_t)d * 4096u, voff, sA + kImgBytes + d * 4096);
#pragma unroll
      for (int d = 0; d < 8; ++d)
        dma16(ldsw + kGradBOff + kImgBytes + (uint32_t)d * 4096u, voff, sB + kImgBytes + d * 4096);
    }
    // k-step s reads A buffer s % 3 and B buffer s % 2
    int s = 0, ia = 0;
    for (; s + 2 < nk; ++s) {
      const int ia1 = ia == kGradABufs - 1 ? 0 : ia + 1, ia2 = ia1 == kGradABufs - 1 ? 0 : ia1 + 1;
      const int ib = (s & 1) * kImgBytes, ib1 = kImgBytes - ib;
      grad_kstep<true, false>(acc, fa, fb, lds + ia * kImgBytes + waveA, lds + ib + waveB,
                              lds + ia1 * kImgBytes + waveA, lds + ib1 + waveB, lane,
                              ldsw + ia2 * kImgBytes, ldsw + kGradBOff + ib, voff,
                              sB + (int64_t)(s + 2) * kImgBytes, sA + (int64_t)(s + 2) * kImgBytes);
      ia = ia1;
    }
    if (s + 1 < nk) {
      const int ia1 = ia == kGradABufs - 1 ? 0 : ia + 1;
      const int ib = (s & 1) * kImgBytes, ib1 = kImgBytes - ib;
      grad_kstep<false, false>(acc, fa, fb, lds + ia * kImgBytes + waveA, lds + ib + waveB,
                               lds + ia1 * kImgBytes + waveA, lds + ib1 + waveB, lane, ldsw, ldsw, voff, sB, sA);
      ia = ia1;
      ++s;
    }
    {
      const int ib = (s & 1) * kImgBytes;
      grad_kstep<false, true>(acc, fa, fb, lds + ia * kImgBytes + waveA, lds + ib + waveB, lds, lds, lane,
                              ldsw, ldsw, voff, sB, sA);
    }
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
struct FinalizeArgs {
  DevicePlan pl; int B; int64_t T; int probe;
  float* g; int ksplit; int64_t n_pad; int H;
  int64_t g_rows;                          // rows per k-split plane of g
  const float* inv_z;                      // 1 / Z_s per computed row (sampled estimator)
  // sampled estimator (Eq. 4): g = c_t (W_s[y_t] - G2 inv_z), G2 = E2 W_s in the second half of
  // g; cr NULL: g is the contraction of the logit gradient itself, in the first half
  const float* cr; const int32_t* ids; const __bf16* W_s; int V;
  float grad_scale; int dh_bf16;
  void* dh_prefix; void* dh_full;
  float* rownorm;
};

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
  for (int h = lane * 4; h < a.H; h += 256) {
    float4 g = *(const float4*)(a.g + r * a.H + h);
    for (int s = 1; s < a.ksplit; ++s) {
      const float4 q = *(const float4*)(a.g + ((int64_t)s * a.g_rows + r) * a.H + h);
      g.x += q.x; g.y += q.y; g.z += q.z; g.w += q.w;
    }
    if (a.ksplit > 1) *(float4*)(a.g + r * a.H + h) = g;
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
}

// ---------------------------------------------------------------------------------------
// Pooled gradients: column sums of g over the window and over the rollout, two levels.
// ---------------------------------------------------------------------------------------
struct PoolArgs {
  DevicePlan pl; int B; int probe; int H;
  const float* g; float* pp; float* pf;   // partials [n_chunks][H]
  float* up; float* uf;                   // [B][H]
};

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
// Workspace layout and the entry point
// ---------------------------------------------------------------------------------------
struct FusedLayout {
  bool use_dma;      // logit passes staged by direct global->LDS loads
  bool single;       // single-sweep scheme (needs use_dma)
  size_t o_wt_img, o_ws_img, o_ht_img, o_hs_img;   // tile images of the logit operands (use_dma)
  int strips1;       // vocabulary strips of the single sweep
  size_t o_ref_t2, o_delta, o_invz, o_mu0t;
  int strips, ksplit;
  int64_t slab_rows, Vp;
  size_t o_plan, o_row_idx, o_row_seq, o_part, o_lse2, o_mu, o_klr, o_rownorm, o_WsT, o_slab, o_g,
      o_pp, o_pf, o_up, o_uf, o_seg, o_racc, o_uc, o_cacc, o_cS, o_cr, o_zy_s, o_zy_t, o_yid, o_dzT_p, o_dzT_f, o_hsT, o_summ, o_cosp, total;
};

static int env_int(const char* name, int dflt) {
  const char* s = getenv(name);
  if (!s || !*s) return dflt;
  const int v = atoi(s);
  return v > 0 ? v : dflt;
}

// Whether any requested output depends on the per-row gradients.  Without one the single
// sweep runs in its statistics-only mode (KL, c, losses, the diagnostics and their summaries):
// no gradient factors are stored, combined or contracted.
static bool needs_gradient(const adwin_opd_problem* p) {
  const bool probe = p->mode == ADWIN_PREFIX_AND_FULL;
  return p->dh_prefix || p->dh_full || p->rho_pooled || p->rho_field || p->dW_prefix || p->dW_full ||
         (probe && (p->batch || (p->candidates && p->n_candidates > 0 &&
                                 (p->cand_rho_pooled || p->cand_rho_field || p->cand_batch))));
}

static FusedLayout fused_layout(const adwin_opd_problem* p, const HostPlan& hp) {
  FusedLayout L;
  const int64_t n_pad = hp.n_pad > 0 ? hp.n_pad : kTileTokens;
  const int vt_total = (p->V + kTileVocab - 1) / kTileVocab;
  L.Vp = (int64_t)vt_total * kTileVocab;
  int strips = env_int("ADWIN_STRIPS", 8);
  if (strips > vt_total) strips = vt_total;
  if (strips > kMaxStrips) strips = kMaxStrips;
  L.strips = strips;
  // the direct-to-LDS logit kernel pipelines at least two k-steps per head
  L.use_dma = !getenv("ADWIN_NO_DMA") && p->H_s >= 2 * kBK && p->H_t >= 2 * kBK;
  L.single = L.use_dma && !getenv("ADWIN_TWO_SWEEP");
  int strips1 = env_int("ADWIN_STRIPS2", 32);
  if (strips1 > vt_total) strips1 = vt_total;
  if (strips1 > kMaxStrips) strips1 = kMaxStrips;
  L.strips1 = strips1;
  const int halves = L.single ? 2 : 1;     // the single sweep stores two factors per logit
  // ... but the gradient GEMM contracts one: the combined logit gradient, or E2 (sampled estimator)
  const int gemm_halves = 1;
  const int h_tiles = (p->H_s + kGradTile - 1) / kGradTile;
  // Rows per slab: a multiple of 8 token tiles (whole rounds of the sweep's workgroups on
  // 256 compute units) between 4,096 and 16,384, chosen so that the gradient GEMM's
  // 256 x 256 output tiles of all slabs fill the fewest rounds; ties go to the larger slab
  // (fewer launches, each of which ends in a partly idle round).
  int64_t slab = 0;
  if (getenv("ADWIN_SLAB_ROWS")) {
    slab = (int64_t)align_up((size_t)env_int("ADWIN_SLAB_ROWS", 8192), kTileTokens);
  } else {
    int64_t best_rounds = -1;
    for (int64_t r = 16384; r >= 4096; r -= 2048) {
      int64_t rounds = 0;
      for (int64_t r0 = 0; r0 < n_pad; r0 += r) {
        const int64_t rows = n_pad - r0 < r ? n_pad - r0 : r;
        rounds += (gemm_halves * (rows / kGradTile) * h_tiles + 255) / 256;
      }
      if (best_rounds < 0 || rounds < best_rounds) { best_rounds = rounds; slab = r; }
    }
  }
  if (slab > n_pad) slab = n_pad;
  L.slab_rows = slab;
  const int64_t tiles = gemm_halves * (slab / kGradTile) * h_tiles;
  int ks = (int)(256 / (tiles > 0 ? tiles : 1));
  const int nk = (int)(L.Vp / kBK);
  if (ks > 16) ks = 16;
  if (ks > nk) ks = nk;
  if (ks < 1) ks = 1;
  L.ksplit = ks;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
  L.o_plan = take(PlanBlobLayout(p->B).bytes);
  L.o_row_idx = take(sizeof(int32_t) * (size_t)n_pad);
  L.o_row_seq = take(sizeof(int32_t) * (size_t)n_pad);
  L.o_part = take(sizeof(float) * 5 * (size_t)(strips > strips1 ? strips : strips1) * (size_t)n_pad);
  L.o_ref_t2 = take(sizeof(float) * (size_t)n_pad);
  L.o_delta = take(sizeof(float) * (size_t)n_pad);
  L.o_mu0t = take((L.single && p->estimator != ADWIN_EST_SAMPLED)
                      ? sizeof(float) * (size_t)vt_total * (size_t)slab : 0);
  L.o_invz = take(sizeof(float) * (size_t)n_pad);
  L.o_lse2 = take(sizeof(float) * (size_t)n_pad);
  L.o_mu = take(sizeof(float) * (size_t)n_pad);
  L.o_klr = take(sizeof(float) * (size_t)n_pad);
  L.o_rownorm = take(sizeof(float) * (size_t)n_pad);
  L.o_WsT = take(2 * (size_t)h_tiles * kGradTile * (size_t)L.Vp);
  L.o_wt_img = take(L.use_dma ? 2 * (size_t)L.Vp * (size_t)p->H_t : 0);
  L.o_ws_img = take(L.use_dma ? 2 * (size_t)L.Vp * (size_t)p->H_s : 0);
  L.o_ht_img = take(L.use_dma ? 2 * (size_t)n_pad * (size_t)p->H_t : 0);
  L.o_hs_img = take(L.use_dma ? 2 * (size_t)n_pad * (size_t)p->H_s : 0);
  // statistics-only calls (no output depends on the gradients) need neither the slab nor g
  const bool need_g = needs_gradient(p) || !L.single;
  L.o_slab = take(need_g ? 2 * (size_t)halves * (size_t)slab * (size_t)L.Vp : 0);
  L.o_g = take(need_g ? sizeof(float) * (size_t)ks * (size_t)halves * (size_t)n_pad * (size_t)p->H_s : 0);
  const size_t nch = (size_t)(hp.n_chunks > 0 ? hp.n_chunks : 1);
  L.o_pp = take(sizeof(float) * nch * (size_t)p->H_s);
  L.o_pf = take(sizeof(float) * nch * (size_t)p->H_s);
  L.o_up = take(sizeof(float) * (size_t)p->B * (size_t)p->H_s);
  L.o_uf = take(sizeof(float) * (size_t)p->B * (size_t)p->H_s);
  L.o_seg = take(sizeof(double) * 4 * (size_t)p->B);
  L.o_racc = take(sizeof(double) * 4 * (size_t)p->B);
  const size_t kc = (p->candidates && p->n_candidates > 0) ? (size_t)p->n_candidates : 0;
  L.o_uc = take(sizeof(float) * kc * (size_t)p->B * (size_t)p->H_s);
  L.o_cacc = take(sizeof(double) * 4 * kc * (size_t)p->B);
  L.o_cS = take(sizeof(double) * kc * (size_t)p->B);
  L.o_cr = take(sizeof(float) * (size_t)n_pad);
  L.o_zy_s = take(sizeof(float) * (size_t)n_pad);
  L.o_zy_t = take(sizeof(float) * (size_t)n_pad);
  L.o_yid = take(sizeof(int32_t) * (size_t)n_pad);
  const bool head = p->dW_prefix || p->dW_full;       // transposed slab + weighted h_s^T images
  // vocabulary tiles of 256 image rows: the last one may be half used (its upper rows are
  // never written, and their output rows do not exist)
  const size_t v_img = align_up((size_t)L.Vp, (size_t)kGradTile);
  L.o_dzT_p = take(p->dW_prefix ? 2 * (size_t)slab * v_img : 0);
  L.o_dzT_f = take(p->dW_full ? 2 * (size_t)slab * v_img : 0);
  L.o_hsT = take(head ? 2 * (size_t)h_tiles * kGradTile * (size_t)slab : 0);
  L.o_cosp = take((p->dW_prefix && p->dW_full) ? sizeof(double) * 3 * kCosineBlocks : 0);
  L.o_summ = take((p->t_first_reject || p->t_logp_mean || p->cand_loss_share)
                      ? sizeof(double) * (size_t)p->B * kSummarySlots : 0);
  L.total = o;
  return L;
}

static void launch_grad(const GradArgs& ga, const FusedLayout& L, hipStream_t stream) {
  grad_gemm_kernel<<<(unsigned)(ga.row_tiles * ga.h_tiles * L.ksplit), 256, kGradLds, stream>>>(ga);
}

static int check_problem(const adwin_opd_problem* p) {
  if (!p) return ADWIN_E_NULL;
  if (p->struct_bytes != sizeof(adwin_opd_problem)) return ADWIN_E_MODE;
  int st = validate_ragged(p->T, p->B, p->offsets, p->window);
  if (st != ADWIN_OK) return st;
  if (p->V <= 0 || (p->V & 7) || p->H_s <= 0 || (p->H_s % kBK) || p->H_t <= 0 || (p->H_t % kBK))
    return ADWIN_E_SHAPE;
  if (p->mode != ADWIN_PREFIX_ONLY && p->mode != ADWIN_PREFIX_AND_FULL) return ADWIN_E_MODE;
  if (p->reduction < ADWIN_RED_SEQ_MEAN || p->reduction > ADWIN_RED_TOKEN_MEAN) return ADWIN_E_MODE;
  if (p->dh_dtype != ADWIN_DT_BF16 && p->dh_dtype != ADWIN_DT_F32) return ADWIN_E_MODE;
  if (p->estimator != ADWIN_EST_EXPECTED && p->estimator != ADWIN_EST_SAMPLED) return ADWIN_E_MODE;
  if (p->n_candidates < 0 || p->n_candidates > ADWIN_MAX_CANDIDATES) return ADWIN_E_SHAPE;
  if (p->candidates && p->n_candidates > 0) {
    if (p->mode != ADWIN_PREFIX_AND_FULL) return ADWIN_E_MODE;
    for (int k = 0; k < p->n_candidates; ++k)
      if (p->candidates[k] <= 0) return ADWIN_E_WINDOW;
  }
  if (p->t_first_reject && !p->t_rank) return ADWIN_E_NULL;
  if (p->t_first_reject && p->topk <= 0) return ADWIN_E_SHAPE;
  if (p->t_logp_mean && !p->t_logp) return ADWIN_E_NULL;
  if (p->cand_loss_share && !(p->candidates && p->n_candidates > 0)) return ADWIN_E_NULL;
  return ADWIN_OK;
}

static hipError_t ensure_lds_opt_in() {
  if (!first_use_on_device(0)) return hipSuccess;
  hipError_t e;
  e = hipFuncSetAttribute((const void*)logit_pass_kernel<false>,
                          hipFuncAttributeMaxDynamicSharedMemorySize, kLogitLds);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute((const void*)logit_pass_kernel<true>,
                          hipFuncAttributeMaxDynamicSharedMemorySize, kLogitLds);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute((const void*)logit_pass_dma_kernel<kModeStats>,
                          hipFuncAttributeMaxDynamicSharedMemorySize, kDmaLds);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute((const void*)logit_pass_dma_kernel<kModeDz>,
                          hipFuncAttributeMaxDynamicSharedMemorySize, kDmaLds);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute((const void*)logit_pass_dma_kernel<kModeSingle>,
                          hipFuncAttributeMaxDynamicSharedMemorySize, kDmaLds);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute((const void*)logit_pass_dma_kernel<kModeSingleDiag>,
                          hipFuncAttributeMaxDynamicSharedMemorySize, kDmaLds);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute((const void*)logit_pass_dma_kernel<kModeSingleE2>,
                          hipFuncAttributeMaxDynamicSharedMemorySize, kDmaLds);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute((const void*)logit_pass_dma_kernel<kModeSingleE2Diag>,
                          hipFuncAttributeMaxDynamicSharedMemorySize, kDmaLds);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute((const void*)logit_pass_dma_kernel<kModeSingleFwd>,
                          hipFuncAttributeMaxDynamicSharedMemorySize, kDmaLds);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute((const void*)logit_pass_dma_kernel<kModeSingleFwdDiag>,
                          hipFuncAttributeMaxDynamicSharedMemorySize, kDmaLds);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute((const void*)grad_gemm_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                          kGradLds);
  if (e != hipSuccess) return e;
  return hipSuccess;
}

}  // namespace adwin

using namespace adwin;

extern "C" int adwin_opd_workspace_bytes(const adwin_opd_problem* p, size_t* bytes) {
  if (!bytes) return ADWIN_E_NULL;
  int st = check_problem(p);
  if (st != ADWIN_OK) return st;
  HostPlan hp = make_host_plan(p->T, p->B, p->offsets, p->window,
                               p->mode == ADWIN_PREFIX_AND_FULL, p->reduction, nullptr);
  *bytes = fused_layout(p, hp).total;
  return ADWIN_OK;
}

extern "C" int adwin_opd_fused_launch_info(const adwin_opd_problem* p, int64_t info[4]) {
  if (!info) return ADWIN_E_NULL;
  int st = check_problem(p);
  if (st != ADWIN_OK) return st;
  HostPlan hp = make_host_plan(p->T, p->B, p->offsets, p->window,
                               p->mode == ADWIN_PREFIX_AND_FULL, p->reduction, nullptr);
  FusedLayout L = fused_layout(p, hp);
  info[0] = hp.n_rows;
  info[1] = hp.n_pad;
  info[2] = L.slab_rows;
  info[3] = hp.n_pad > 0 ? (hp.n_pad + L.slab_rows - 1) / L.slab_rows : 0;
  return ADWIN_OK;
}

static int fused_impl(const adwin_opd_problem* p, void* workspace, size_t workspace_bytes,
                      void* hip_stream, PhaseTimer* timer) {
  int st = check_problem(p);
  if (st != ADWIN_OK) return st;
  if (!p->W_s || !p->W_t) return ADWIN_E_NULL;
  if (p->T > 0 && (!p->h_s || !p->h_t)) return ADWIN_E_NULL;
  const uintptr_t al = (uintptr_t)p->h_s | (uintptr_t)p->h_t | (uintptr_t)p->W_s |
                       (uintptr_t)p->W_t | (uintptr_t)p->dh_prefix | (uintptr_t)p->dh_full;
  if (al & 15) return ADWIN_E_ALIGN;
  const int probe = p->mode == ADWIN_PREFIX_AND_FULL;
  std::vector<unsigned char> blob;
  HostPlan hp = make_host_plan(p->T, p->B, p->offsets, p->window, probe, p->reduction, &blob);
  FusedLayout L = fused_layout(p, hp);
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < L.total)
    return ADWIN_E_WORKSPACE;
  const bool diag = p->t_entropy || p->t_rank;          // need the diagnostics sweep
  const bool sampled = p->estimator == ADWIN_EST_SAMPLED;
  // the diagnostics and the sampled estimator ride on the single-sweep kernels
  const bool head = p->dW_prefix || p->dW_full;
  const bool need_g = needs_gradient(p) || !L.single;   // the statistics-only mode is a single-sweep mode
  if ((diag || p->t_logp || sampled || head) && !L.single) return ADWIN_E_MODE;
  if (sampled && !p->ids) return ADWIN_E_NULL;
  if (p->dW_full && p->mode != ADWIN_PREFIX_AND_FULL) return ADWIN_E_MODE;
  if (((uintptr_t)p->dW_prefix | (uintptr_t)p->dW_full) & 15) return ADWIN_E_ALIGN;
  hipStream_t stream = (hipStream_t)hip_stream;
  unsigned char* ws = (unsigned char*)workspace;
  ADWIN_HIP_TRY(ensure_lds_opt_in());

  PhaseScope* scope = new PhaseScope(timer, ADWIN_PHASE_SETUP);
  struct ScopeGuard { PhaseScope*& s; ~ScopeGuard() { delete s; } } guard{scope};
  auto phase = [&](int ph) { delete scope; scope = new PhaseScope(timer, ph); };
  ADWIN_HIP_TRY(launch_upload(ws + L.o_plan, blob.data(), blob.size(), stream));
  DevicePlan pl = device_plan_at(ws + L.o_plan, p->B, (int32_t*)(ws + L.o_row_idx),
                                 (int32_t*)(ws + L.o_row_seq));
  float* klr = (float*)(ws + L.o_klr);
  float* rownorm = (float*)(ws + L.o_rownorm);
  float* gws = (float*)(ws + L.o_g);
  double* seg = (double*)(ws + L.o_seg);
  const int64_t n_pad = hp.n_pad;

  ADWIN_HIP_TRY(launch_fill_u32(p->status_dev, 1, 0u, stream));
  if (!probe) {   // rows outside the windows report zero KL, cost and diagnostics
    ADWIN_HIP_TRY(launch_fill_f32(p->kl, p->T, 0.f, stream));
    ADWIN_HIP_TRY(launch_fill_f32(p->c, p->T, 0.f, stream));
    ADWIN_HIP_TRY(launch_fill_f32(p->t_logp, p->T, 0.f, stream));
    ADWIN_HIP_TRY(launch_fill_f32(p->t_entropy, p->T, 0.f, stream));
    ADWIN_HIP_TRY(launch_fill_u32((uint32_t*)p->t_rank, p->T, 0u, stream));
  } else if (!p->ids) {
    ADWIN_HIP_TRY(launch_fill_f32(p->c, p->T, 0.f, stream));
  }

  if (hp.n_rows > 0) {
    ADWIN_HIP_TRY(launch_build_rows(pl, p->B, hp.n_rows, n_pad, stream));
    const int vt_total = (int)(L.Vp / kTileVocab);
    const int n_tiles = (int)(n_pad / kTileTokens);
    // tile images of W_s^T for the gradient GEMM
    const int h_tiles = (p->H_s + kGradTile - 1) / kGradTile;
    if (need_g) {
      dim3 g((unsigned)(L.Vp / kBK), (unsigned)h_tiles);
      wst_image_kernel<<<g, 256, 0, stream>>>((const uint16_t*)p->W_s, (uint16_t*)(ws + L.o_WsT), p->V,
                                              p->H_s, (int)(L.Vp / kBK));
      ADWIN_HIP_TRY(hipGetLastError());
    }
    const bool use_dma = L.use_dma;
    if (use_dma) {
      // tile images of the logit operands: vocabulary tiles of 128 rows (zero beyond V),
      // token tiles of 256 computed rows gathered through row_idx
      RowImageArgs ia;
      ia.row_idx = nullptr; ia.n_rows = p->V; ia.th = kTileVocab;
      ia.src = (const uint4*)p->W_t; ia.img = (uint4*)(ws + L.o_wt_img); ia.H = p->H_t; ia.nk = p->H_t / kBK;
      row_image_kernel<<<dim3((unsigned)ia.nk, (unsigned)vt_total), 256, 0, stream>>>(ia);
      ADWIN_HIP_TRY(hipGetLastError());
      ia.src = (const uint4*)p->W_s; ia.img = (uint4*)(ws + L.o_ws_img); ia.H = p->H_s; ia.nk = p->H_s / kBK;
      row_image_kernel<<<dim3((unsigned)ia.nk, (unsigned)vt_total), 256, 0, stream>>>(ia);
      ADWIN_HIP_TRY(hipGetLastError());
      ia.row_idx = pl.row_idx; ia.n_rows = n_pad; ia.th = kTileTokens;
      ia.src = (const uint4*)p->h_t; ia.img = (uint4*)(ws + L.o_ht_img); ia.H = p->H_t; ia.nk = p->H_t / kBK;
      row_image_kernel<<<dim3((unsigned)ia.nk, (unsigned)n_tiles), 256, 0, stream>>>(ia);
      ADWIN_HIP_TRY(hipGetLastError());
      ia.src = (const uint4*)p->h_s; ia.img = (uint4*)(ws + L.o_hs_img); ia.H = p->H_s; ia.nk = p->H_s / kBK;
      row_image_kernel<<<dim3((unsigned)ia.nk, (unsigned)n_tiles), 256, 0, stream>>>(ia);
      ADWIN_HIP_TRY(hipGetLastError());
    }
    LogitPassArgs la;
    la.h_s = (const __bf16*)p->h_s; la.h_t = (const __bf16*)p->h_t;
    la.W_s = (const __bf16*)p->W_s; la.W_t = (const __bf16*)p->W_t;
    la.H_s = p->H_s; la.H_t = p->H_t; la.V = p->V;
    la.row_idx = pl.row_idx; la.n_pad = n_pad;
    la.vt_total = vt_total;
    la.part = (float*)(ws + L.o_part);
    la.lse2 = (const float*)(ws + L.o_lse2); la.mu = (const float*)(ws + L.o_mu);
    la.slab = (__bf16*)(ws + L.o_slab); la.Vp = L.Vp;
    la.ref_s2 = (const float*)(ws + L.o_lse2); la.ref_t2 = (const float*)(ws + L.o_ref_t2);
    la.mu0 = (const float*)(ws + L.o_mu); la.e2_off = 0;
    la.mu0t = (L.single && !sampled && need_g) ? (float*)(ws + L.o_mu0t) : nullptr; la.mu0t_stride = L.slab_rows;
    la.tg = env_int("ADWIN_TG", 4);
    la.Wt_img = (const char*)(ws + L.o_wt_img); la.Ws_img = (const char*)(ws + L.o_ws_img);
    la.ht_img = (const char*)(ws + L.o_ht_img); la.hs_img = (const char*)(ws + L.o_hs_img);
    MergeArgs m;
    m.part = la.part; m.strips = L.strips; m.n_pad = n_pad; m.n_rows = hp.n_rows;
    m.row_idx = pl.row_idx;
    m.h_s = la.h_s; m.h_t = la.h_t; m.W_s = la.W_s; m.W_t = la.W_t;
    m.H_s = p->H_s; m.H_t = p->H_t; m.V = p->V; m.ids = p->ids;
    m.lse2 = (float*)(ws + L.o_lse2); m.mu = (float*)(ws + L.o_mu); m.klr = klr;
    m.kl = p->kl; m.c = p->c; m.status = p->status_dev;
    m.diag = diag ? 1 : 0; m.t_logp = p->t_logp; m.t_entropy = p->t_entropy; m.t_rank = p->t_rank;
    m.cr = sampled ? (float*)(ws + L.o_cr) : nullptr;
    GradArgs ga;
    ga.slab = la.slab; ga.WsT = (const __bf16*)(ws + L.o_WsT); ga.nk_total = (int)(L.Vp / kBK);
    ga.g = gws; ga.H = p->H_s; ga.h_tiles = h_tiles; ga.ksplit = L.ksplit;
    ga.out_rows = (int64_t)1 << 62; ga.accumulate = 0;
    if (L.single) {
      // Single sweep.  (1) online statistics of vocabulary tile 0 give each row its fixed
      // references; (2) per row slab: one sweep over the vocabulary producing the strip sums
      // and the two gradient factors, then one GEMM of both factors with W_s; (3) merge.
      la.tile0 = 0; la.n_tiles = n_tiles; la.strips = 1; la.vt_total = 1;
      {
        const int groups = (n_tiles + la.tg - 1) / la.tg;
        logit_pass_dma_kernel<kModeStats><<<(unsigned)(groups * la.tg), 256, kDmaLds, stream>>>(la);
        ADWIN_HIP_TRY(hipGetLastError());
        if (p->ids || diag) {      // without ids: id -1 on every row, which the diagnostics sweep expects
          TokenLogitArgs ta;
          ta.row_idx = pl.row_idx; ta.ids = p->ids;
          ta.h_s = la.h_s; ta.W_s = la.W_s; ta.h_t = la.h_t; ta.W_t = la.W_t;
          ta.H_s = p->H_s; ta.H_t = p->H_t; ta.V = p->V; ta.n_pad = n_pad;
          ta.zy_s = (float*)(ws + L.o_zy_s); ta.zy_t = (float*)(ws + L.o_zy_t);
          ta.yid = (int32_t*)(ws + L.o_yid);
          token_logit_kernel<<<(unsigned)((n_pad + 3) / 4), 256, 0, stream>>>(ta);
          ADWIN_HIP_TRY(hipGetLastError());
        }
        make_refs_kernel<<<(unsigned)((n_pad + 255) / 256), 256, 0, stream>>>(
            la.part, n_pad, (const float*)(ws + L.o_zy_s), (const float*)(ws + L.o_zy_t),
            p->ids ? (const int32_t*)(ws + L.o_yid) : nullptr, (float*)(ws + L.o_lse2),
            (float*)(ws + L.o_ref_t2), (float*)(ws + L.o_mu));
        ADWIN_HIP_TRY(hipGetLastError());
      }
      la.vt_total = vt_total; la.strips = L.strips1;
      la.zy_t = (const float*)(ws + L.o_zy_t); la.yid = (const int32_t*)(ws + L.o_yid);
      ga.g_rows = 2 * n_pad; ga.half_off = n_pad;
      for (int64_t r0 = 0; r0 < n_pad; r0 += L.slab_rows) {
        const int64_t rows = (n_pad - r0 < L.slab_rows) ? n_pad - r0 : L.slab_rows;
        la.tile0 = (int)(r0 / kTileTokens); la.n_tiles = (int)(rows / kTileTokens);
        la.e2_off = rows * L.Vp;
        const int groups = (la.n_tiles + la.tg - 1) / la.tg;
        phase(ADWIN_PHASE_STATS);
        const unsigned sweep_grid = (unsigned)(groups * la.tg * L.strips1);
        if (!need_g && diag) logit_pass_dma_kernel<kModeSingleFwdDiag><<<sweep_grid, 256, kDmaLds, stream>>>(la);
        else if (!need_g) logit_pass_dma_kernel<kModeSingleFwd><<<sweep_grid, 256, kDmaLds, stream>>>(la);
        else if (sampled && diag) logit_pass_dma_kernel<kModeSingleE2Diag><<<sweep_grid, 256, kDmaLds, stream>>>(la);
        else if (sampled) logit_pass_dma_kernel<kModeSingleE2><<<sweep_grid, 256, kDmaLds, stream>>>(la);
        else if (diag) logit_pass_dma_kernel<kModeSingleDiag><<<sweep_grid, 256, kDmaLds, stream>>>(la);
        else logit_pass_dma_kernel<kModeSingle><<<sweep_grid, 256, kDmaLds, stream>>>(la);
        ADWIN_HIP_TRY(hipGetLastError());
        // this slab's rows are complete: KL_t, c_t, mu; then the logit gradient proper
        phase(ADWIN_PHASE_MERGE);
        MergeSingleArgs ms;
        ms.m = m; ms.m.strips = L.strips1;
        ms.ref_s2 = la.ref_s2; ms.ref_t2 = la.ref_t2;
        ms.mu_out = (float*)(ws + L.o_delta); ms.inv_z = (float*)(ws + L.o_invz);
        ms.row0 = r0; ms.rows = rows;
        merge_single_kernel<<<(unsigned)((rows + 3) / 4), 256, 0, stream>>>(ms);
        ADWIN_HIP_TRY(hipGetLastError());
        if (!need_g) continue;
        ga.slab_row0 = r0;
        ga.row_tiles = (int)(rows / kGradTile);
        CombineArgs ca;
        ca.slab = (uint4*)la.slab; ca.e2_vec = la.e2_off / 8;
        ca.mu = ms.mu_out; ca.inv_z = ms.inv_z; ca.row0 = r0; ca.nk = ga.nk_total;
        ca.mu0t = la.mu0t; ca.mu0t_stride = la.mu0t_stride;
        ca.dzT_p = p->dW_prefix ? (uint4*)(ws + L.o_dzT_p) : nullptr;
        ca.dzT_f = p->dW_full ? (uint4*)(ws + L.o_dzT_f) : nullptr;
        ca.nkr = (int)(rows / kBK); ca.pl = pl; ca.n_rows = hp.n_rows; ca.grad_scale = p->grad_scale;
        ca.cr = (const float*)(ws + L.o_cr); ca.yid = (const int32_t*)(ws + L.o_yid);
        const dim3 cgrid((unsigned)ga.nk_total, (unsigned)ga.row_tiles);
        if (sampled) {       // contract the E2 factor; c_t and W_s[y_t] enter in finalize_kernel
          ga.slab = la.slab + la.e2_off;
          ga.half_tiles = 0;                       // output rows in the second half of g
          if (head) {        // the transposed operand of the head-weight GEMMs; the slab stays as it is
            phase(ADWIN_PHASE_DZ);
            combine_kernel<true, true><<<cgrid, 256, 0, stream>>>(ca);
            ADWIN_HIP_TRY(hipGetLastError());
          }
        } else {
          phase(ADWIN_PHASE_DZ);
          if (head) combine_kernel<true><<<cgrid, 256, 0, stream>>>(ca);
          else combine_kernel<false><<<cgrid, 256, 0, stream>>>(ca);
          ADWIN_HIP_TRY(hipGetLastError());
          ga.half_tiles = ga.row_tiles;            // output rows in the first half of g
        }
        phase(ADWIN_PHASE_GRAD);
        launch_grad(ga, L, stream);
        ADWIN_HIP_TRY(hipGetLastError());
        if (head) {
          // head-weight gradient of this slab: dW += dz^T (w h_s), k = the slab's rows
          GradArgs wa = ga;
          wa.WsT = (const __bf16*)(ws + L.o_hsT);
          wa.nk_total = (int)(rows / kBK);
          wa.H = p->H_s; wa.h_tiles = h_tiles; wa.ksplit = 1;
          wa.slab_row0 = 0; wa.row_tiles = (int)((L.Vp + kGradTile - 1) / kGradTile); wa.half_tiles = wa.row_tiles;
          wa.half_off = 0; wa.g_rows = 0; wa.out_rows = p->V; wa.accumulate = r0 > 0;
          HstImageArgs ha;
          ha.h_s = (const uint16_t*)p->h_s; ha.row_idx = pl.row_idx;
          ha.row0 = r0; ha.H = p->H_s; ha.nkr = wa.nk_total;
          ha.img = (uint16_t*)(ws + L.o_hsT);
          hst_image_kernel<<<dim3((unsigned)ha.nkr, (unsigned)h_tiles), 256, 0, stream>>>(ha);
          ADWIN_HIP_TRY(hipGetLastError());
          for (int which = 0; which < 2; ++which) {
            float* out = which == 0 ? p->dW_prefix : p->dW_full;
            if (!out) continue;
            wa.slab = (const __bf16*)(ws + (which == 0 ? L.o_dzT_p : L.o_dzT_f));
            wa.g = out;
            grad_gemm_kernel<<<(unsigned)(wa.row_tiles * wa.h_tiles), 256, kGradLds, stream>>>(wa);
            ADWIN_HIP_TRY(hipGetLastError());
          }
        }
      }
    } else {
      // Two sweeps: statistics over all token tiles, merge, then per row slab the dz sweep
      // and its GEMM with W_s.
      phase(ADWIN_PHASE_STATS);
      {
        la.tile0 = 0; la.n_tiles = n_tiles; la.strips = L.strips;
        const int groups = (n_tiles + la.tg - 1) / la.tg;
        if (use_dma)
          logit_pass_dma_kernel<kModeStats><<<(unsigned)(groups * la.tg * L.strips), 256, kDmaLds, stream>>>(la);
        else
          logit_pass_kernel<false><<<(unsigned)(groups * la.tg * L.strips), 256, kLogitLds, stream>>>(la);
        ADWIN_HIP_TRY(hipGetLastError());
      }
      phase(ADWIN_PHASE_MERGE);
      merge_stats_kernel<<<(unsigned)((n_pad + 3) / 4), 256, 0, stream>>>(m);
      ADWIN_HIP_TRY(hipGetLastError());
      const int strips2 = L.strips1;
      ga.g_rows = n_pad; ga.half_off = 0;
      for (int64_t r0 = 0; r0 < n_pad; r0 += L.slab_rows) {
        const int64_t rows = (n_pad - r0 < L.slab_rows) ? n_pad - r0 : L.slab_rows;
        la.tile0 = (int)(r0 / kTileTokens); la.n_tiles = (int)(rows / kTileTokens);
        la.strips = strips2;
        const int groups = (la.n_tiles + la.tg - 1) / la.tg;
        phase(ADWIN_PHASE_DZ);
        if (use_dma)
          logit_pass_dma_kernel<kModeDz><<<(unsigned)(groups * la.tg * strips2), 256, kDmaLds, stream>>>(la);
        else
          logit_pass_kernel<true><<<(unsigned)(groups * la.tg * strips2), 256, kLogitLds, stream>>>(la);
        ADWIN_HIP_TRY(hipGetLastError());
        phase(ADWIN_PHASE_GRAD);
        ga.slab_row0 = r0;
        ga.row_tiles = (int)(rows / kGradTile); ga.half_tiles = ga.row_tiles;
        launch_grad(ga, L, stream);
        ADWIN_HIP_TRY(hipGetLastError());
      }
    }
  }
  if (hp.n_rows == 0) {     // nothing computed: the head-weight gradients are zero
    ADWIN_HIP_TRY(launch_fill_f32(p->dW_prefix, (int64_t)p->V * p->H_s, 0.f, stream));
    ADWIN_HIP_TRY(launch_fill_f32(p->dW_full, (int64_t)p->V * p->H_s, 0.f, stream));
  }
  // finalize over every packed row (also zero-fills rows outside the windows)
  phase(ADWIN_PHASE_REDUCE);
  if (p->T > 0 && need_g) {
    FinalizeArgs f;
    f.pl = pl; f.B = p->B; f.T = p->T; f.probe = probe;
    f.g = gws; f.ksplit = L.ksplit; f.n_pad = n_pad; f.H = p->H_s;
    f.g_rows = L.single ? 2 * n_pad : n_pad;
    f.inv_z = L.single ? (const float*)(ws + L.o_invz) : nullptr;
    f.cr = (L.single && p->estimator == ADWIN_EST_SAMPLED) ? (const float*)(ws + L.o_cr) : nullptr;
    f.ids = p->ids; f.W_s = (const __bf16*)p->W_s; f.V = p->V;
    f.grad_scale = p->grad_scale; f.dh_bf16 = p->dh_dtype == ADWIN_DT_BF16;
    f.dh_prefix = p->dh_prefix; f.dh_full = p->dh_full; f.rownorm = rownorm;
    finalize_kernel<<<(unsigned)((p->T + 3) / 4), 256, 0, stream>>>(f);
    ADWIN_HIP_TRY(hipGetLastError());
  }
  ADWIN_HIP_TRY(launch_segment_sums(pl, p->B, probe, klr, need_g ? rownorm : nullptr, seg, p->loss_prefix,
                                    p->loss_full, stream));
  PoolArgs pa;
  pa.pl = pl; pa.B = p->B; pa.probe = probe; pa.H = p->H_s; pa.g = gws;
  pa.pp = (float*)(ws + L.o_pp); pa.pf = (float*)(ws + L.o_pf);
  pa.up = (float*)(ws + L.o_up); pa.uf = (float*)(ws + L.o_uf);
  if (probe && need_g) {
    const unsigned hy = (unsigned)((p->H_s + 255) / 256);
    if (hp.n_chunks > 0) {
      pool_partial_kernel<<<dim3((unsigned)hp.n_chunks, hy), 256, 0, stream>>>(pa);
      ADWIN_HIP_TRY(hipGetLastError());
    }
    pool_final_kernel<<<dim3((unsigned)p->B, hy), 256, 0, stream>>>(pa);
    ADWIN_HIP_TRY(hipGetLastError());
  }
  BatchArgs b{};
  b.pl = pl; b.B = p->B; b.H = need_g ? p->H_s : 0; b.probe = probe;
  b.zero_grad = (p->grad_scale == 0.f) || !need_g;
  b.seg = seg; b.up = pa.up; b.uf = pa.uf; b.racc = (double*)(ws + L.o_racc);
  b.rho_pooled = p->rho_pooled; b.rho_field = p->rho_field; b.batch = p->batch;
  b.n_out = p->n_out; b.n_adm_out = p->n_adm_out; b.n_adm = hp.n_adm;
  ADWIN_HIP_TRY(launch_alignment_and_batch(b, stream));
  if (probe && need_g && p->candidates && p->n_candidates > 0) {
    CandArgs ca{};
    ca.pl = pl; ca.B = p->B; ca.H = p->H_s; ca.K = p->n_candidates;
    ca.reduction = p->reduction; ca.zero_grad = (p->grad_scale == 0.f);
    for (int k = 0; k < ca.K; ++k) {
      ca.L[k] = p->candidates[k];
      int64_t nadm = 0;
      for (int32_t i = 0; i < p->B; ++i) {
        const int64_t len = p->offsets[i + 1] - p->offsets[i];
        nadm += ca.L[k] < len ? (int64_t)ca.L[k] : len;
      }
      ca.inv_nadm[k] = nadm > 0 ? 1.0 / (double)nadm : 0.0;
    }
    ca.g = gws; ca.pf = pa.pf; ca.uf = pa.uf; ca.rownorm = rownorm; ca.seg = seg;
    ca.uc = (float*)(ws + L.o_uc); ca.cacc = (double*)(ws + L.o_cacc); ca.cS = (double*)(ws + L.o_cS);
    ca.rho_pooled = p->cand_rho_pooled; ca.rho_field = p->cand_rho_field; ca.batch = p->cand_batch;
    ADWIN_HIP_TRY(launch_candidate_audit(ca, stream));
  }
  // alignment of the two objectives in the LM-head parameter block: batch[6]
  if (p->dW_prefix && p->dW_full && p->batch)
    ADWIN_HIP_TRY(launch_cosine(p->dW_prefix, p->dW_full, (int64_t)p->V * p->H_s,
                                (double*)(ws + L.o_cosp), p->batch + 6, stream));
  if (p->t_first_reject || p->t_logp_mean || p->cand_loss_share) {
    SummaryArgs sa{};
    sa.pl = pl; sa.B = p->B; sa.probe = probe; sa.topk = p->topk;
    sa.K = p->cand_loss_share ? p->n_candidates : 0;
    for (int k = 0; k < sa.K; ++k) sa.L[k] = p->candidates[k];
    sa.t_rank = p->t_rank; sa.t_logp = p->t_logp;
    sa.kl = klr;             // per computed row = per packed row in the full-rollout mode
    sa.acc = (double*)(ws + L.o_summ);
    sa.first_reject = p->t_first_reject; sa.logp_mean = p->t_logp_mean; sa.loss_share = p->cand_loss_share;
    ADWIN_HIP_TRY(launch_summaries(sa, stream));
  }
  return ADWIN_OK;
}

extern "C" int adwin_opd_fused(const adwin_opd_problem* p, void* workspace, size_t workspace_bytes,
                               void* hip_stream) {
  return fused_impl(p, workspace, workspace_bytes, hip_stream, nullptr);
}

extern "C" int adwin_opd_fused_profile(const adwin_opd_problem* p, void* workspace,
                                       size_t workspace_bytes, void* hip_stream, float* phase_ms) {
  if (!phase_ms) return ADWIN_E_NULL;
  PhaseTimer timer((hipStream_t)hip_stream);
  int st = fused_impl(p, workspace, workspace_bytes, hip_stream, &timer);
  if (st != ADWIN_OK) return st;
  ADWIN_HIP_TRY(timer.collect(phase_ms, ADWIN_N_PHASES));
  return ADWIN_OK;
}
