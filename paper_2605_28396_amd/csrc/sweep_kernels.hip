// Fused path, first half: LM-head projections on bf16 MFMA and everything that is taken
// from the logits while they sit in registers -- full-vocabulary log-sum-exp, per-token
// reverse KL (Eq. 2 at token level) and the factors of the logit gradient (Eq. 4 in
// expectation, App. A.1).  The logits themselves are never written anywhere.
//
// Single sweep (the default): per-row references are fixed in advance (online statistics
// of vocabulary tile 0 and the sampled token's logits), so one pass over the vocabulary
// yields the sums Z_s, A = sum e_s (z_s - z_t), Z_t and two bf16 gradient factors
// D = (z_s - z_t) - mu0 and E2 = e_s per logit, written as tile images into a bounded row
// slab; the merge gives lse, mu, KL_t, c_t per row, and the combine pass (grad_kernels.hip)
// turns the factors into dz = p_s ((z_s - z_t) - mu).
// Two sweeps (fallback): running-max statistics, merge, then the logits again for dz.
//
// For a 256-token tile a workgroup walks vocabulary tiles of 128; per tile two MFMA GEMMs
// (teacher, then student) into fp32 accumulators, then the epilogue on the registers.
// MFMA operand roles: v_mfma_f32_32x32x16_bf16 computes D[i][j] += sum_k A[i][k] B[k][j]
// with i in registers and j = lane % 32.  A = W tile (i = vocabulary) and B = h tile
// (j = token), so each lane owns one token column and the reduction over the vocabulary
// runs down its own registers with no cross-lane traffic.
// A lane holds rows i = 8 (e / 4) + 4 (lane / 32) + e % 4 of a 32 x 32 block, e = 0..15.  The
// W tiles are staged with their rows permuted inside every group of 32 (entry_of_tile_row), so
// that these are 16 consecutive vocabulary entries, 16 (lane / 32) + e: a lane then owns 32
// consecutive bytes of a slab row per block and writes them with two 16-byte stores, where the
// natural order gives it four separate 8-byte pieces.
#include "fused_shared.h"

namespace adwin {

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

// Row order of the staged W tiles: tile row 8 q + 4 h + r of a group of 32 holds vocabulary entry
// 16 h + 4 q + r of the group (q = 0..3, h = 0..1, r = 0..3).
__device__ __forceinline__ int entry_of_tile_row(int i) {
  return (i & ~31) + 16 * ((i >> 2) & 1) + 4 * ((i >> 3) & 3) + (i & 3);
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

// ---------------------------------------------------------------------------------------
// Logit passes
// ---------------------------------------------------------------------------------------

// Running per-token statistics held by one lane for its two token columns.
struct LaneStats { float m_s[2], Z_s[2], A_s[2], m_t[2], Z_t[2]; };

// Element e of block fm is vocabulary entry v0 + fm*32 + 16*(lane/32) + e.
// Online update of (m_s, Z_s, A, m_t, Z_t) with one 128 x 64 logit tile per wave.
__device__ __forceinline__ void stats_epilogue(const f32x16 (&zs)[4][2], const f32x16 (&zt)[4][2],
                                               LaneStats& st, int v0, int V, bool tail, int lane) {
  const int vlane = v0 + 16 * (lane >> 5);
#pragma unroll
  for (int fn = 0; fn < 2; ++fn) {
    float mxs = st.m_s[fn], mxt = st.m_t[fn];
#pragma unroll
    for (int fm = 0; fm < 4; ++fm)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const bool ok = !tail || (vlane + fm * 32 + e) < V;
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
        const bool ok = !tail || (vlane + fm * 32 + e) < V;
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

// dz = p_s ((z_s - z_t) - mu), rounded to bf16, into rows wrow + fn*32 + lane%32 of the tile.
// Entries with p_s >= kHeavyP are listed for computed row crow + fn*32 + lane%32 and stored as 0.
__device__ __forceinline__ void dz_epilogue(const f32x16 (&zs)[4][2], const f32x16 (&zt)[4][2],
                                            const float (&lse2)[2], const float (&mu)[2], __bf16* blk,
                                            int wrow, int v0, int V, bool tail, int lane,
                                            const HeavyList& heavy, int64_t crow) {
  // chunk c = 4 (fm & 1) + 2 half + p of slab block fm / 2 holds the lane's entries 8 p .. 8 p + 7
  // of block fm; its position in the row is c ^ key = (4 (fm & 1) + p) ^ key2
  const int half = lane >> 5, vlane = v0 + 16 * half, key2 = ((lane >> 1) & 7) ^ (2 * half);
#pragma unroll
  for (int fn = 0; fn < 2; ++fn) {
    __bf16* out = blk + (wrow + fn * 32 + (lane & 31)) * kBK;
#pragma unroll
    for (int fm = 0; fm < 4; ++fm)
#pragma unroll
      for (int p = 0; p < 2; ++p) {
        float d[8];
        const bool in = !tail || vlane + fm * 32 + 8 * p < V;      // V is a multiple of 8
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float s = zs[fm][fn][p * 8 + e], t = zt[fm][fn][p * 8 + e];
          const float pr = fast_exp2(fmaf(s, kLog2e, -lse2[fn]));
          d[e] = in ? pr * ((s - t) - mu[fn]) : 0.f;
          if (__builtin_expect(pr >= kHeavyP && in, 0)) {
            if (heavy_push(heavy, crow + fn * 32 + (lane & 31), vlane + fm * 32 + 8 * p + e)) d[e] = 0.f;
          }
        }
        uint4 o;
        o.x = pack_bf16(d[0], d[1]); o.y = pack_bf16(d[2], d[3]);
        o.z = pack_bf16(d[4], d[5]); o.w = pack_bf16(d[6], d[7]);
        *(uint4*)(out + (fm >> 1) * kSlabBlock + ((((fm & 1) * 4 + p) ^ key2) << 3)) = o;
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

// One accumulator element for vector arithmetic.  The operand constraint keeps the accumulators
// in their registers up to the read: left alone, the register allocator moves blocks of them
// about (and one into scratch memory) during the epilogue, and every reload from scratch waits
// for all the stores in flight.
__device__ __forceinline__ float acc_read(const float& a) {
  float v;
  asm("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
  return v;
}

// The two slab blocks of a logit tile through a buffer descriptor: the lane's offset is one
// 32-bit register and the block, the token column group and the chunk are immediates or
// scalars, so the stores need no 64-bit address registers.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t slab_rsrc(__bf16* blk) {
  // extent: the tile's two blocks; flag word: the raw-buffer setting of the gfx9 family
  // (32-bit data format, no swizzle)
  return __builtin_amdgcn_make_buffer_rsrc(blk, 0, 2 * kImgBytesSlab, 0x00020000);
}
__device__ __forceinline__ void slab_store16(__amdgpu_buffer_rsrc_t r, int lane_off, int block_off, const float (&x)[8]) {
  u32x4 o;
  o.x = pack_bf16(x[0], x[1]); o.y = pack_bf16(x[2], x[3]);
  o.z = pack_bf16(x[4], x[5]); o.w = pack_bf16(x[6], x[7]);
  __builtin_amdgcn_raw_buffer_store_b128(o, r, lane_off, block_off, 0);
}

template <bool TAIL, bool DIAG, bool WRITE_D, bool WRITE_E2>
__device__ __forceinline__ void single_epilogue(const f32x16 (&zs)[4][2], const f32x16 (&zt)[4][2],
                                                LaneSums& sm, const float (&rs2)[2],
                                                const float (&rt2)[2], float (&mu0)[2],
                                                const float (&zyt)[2], const int (&yid)[2],
                                                __bf16* blk, int64_t e2_off, int wrow,
                                                int v0, int V, int lane, float* mu0_out) {
  // lane's entries of block fm: v0 + fm*32 + 16*half + e, e = 0..15; chunk positions as in dz_epilogue
  const int half = lane >> 5, vlane = v0 + 16 * half, key2 = ((lane >> 1) & 7) ^ (2 * half);
  // byte offset of chunk cb of the lane's row (fn = 0, first block): rowb ^ (cb << 4)
  const int rowb = (wrow + (lane & 31)) * kRowBytes + (key2 << 4);
  const __amdgpu_buffer_rsrc_t rd = slab_rsrc(blk), re = slab_rsrc(blk + e2_off);
  float Zs[2], As[2], Zt[2], Bt[2];
  int cnt[2], vy[2];
#pragma unroll
  for (int fn = 0; fn < 2; ++fn) {
    Zs[fn] = sm.Z_s[fn]; As[fn] = sm.A_s[fn]; Zt[fn] = sm.Z_t[fn]; Bt[fn] = sm.B_t[fn];
    cnt[fn] = sm.cnt[fn];
    vy[fn] = yid[fn] - vlane;              // position of the sampled token among this lane's entries
  }
  // first pass over 8 entries of token column fn: sums and the E2 factor
  auto sums8 = [&](int fn, int fm, int p) __attribute__((always_inline)) {
    float e2[8];
    const bool ok = !TAIL || (vlane + fm * 32 + 8 * p) < V;      // V is a multiple of 8
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float s = acc_read(zs[fm][fn][p * 8 + e]), t = acc_read(zt[fm][fn][p * 8 + e]);
      float es = fast_exp2(fmaf(s, kLog2e, -rs2[fn]));
      float et = fast_exp2(fmaf(t, kLog2e, -rt2[fn]));
      float d = s - t;
      if (TAIL && !ok) { es = 0.f; et = 0.f; d = 0.f; }
      Zs[fn] += es;
      As[fn] = fmaf(es, d, As[fn]);
      Zt[fn] += et;
      if (DIAG) {
        Bt[fn] = fmaf(et, t, Bt[fn]);
        cnt[fn] += (t > zyt[fn] && (fm * 32 + 8 * p + e) != vy[fn] && ok) ? 1 : 0;
      }
      e2[e] = es;
    }
    if (WRITE_E2)
      slab_store16(re, rowb ^ (((fm & 1) * 4 + p) << 4), (fm >> 1) * kImgBytesSlab + fn * 32 * kRowBytes, e2);
  };
  // Second factor: D = d - mu0 with mu0 the strip's running mean of d = z_s - z_t under the
  // student weights, this tile included (both half-columns of the row).  A heavy entry
  // dominates the mean of its own tile, so its D is stored small and the correction
  // (mu - mu0) carries its gradient: the rounding of both factors stays proportional to
  // p_s |d - mu| even when the row is peaked and the first vocabulary entries say nothing
  // about mu.  The masked entries of a tail tile have E2 = 0; their D is immaterial.
  auto mean_of = [&](int fn) __attribute__((always_inline)) {
    const float Zr = Zs[fn] + __shfl_xor(Zs[fn], 32, 64), Ar = As[fn] + __shfl_xor(As[fn], 32, 64);
    if (Zr > 0.f) mu0[fn] = Ar / Zr;
    if (mu0_out && lane < 32) mu0_out[fn * 32 + lane] = mu0[fn];
    return mu0[fn];
  };
  auto factor8 = [&](int fn, int fm, int p, float m0) __attribute__((always_inline)) {
    float dd[8];
#pragma unroll
    for (int e = 0; e < 8; ++e)
      dd[e] = (acc_read(zs[fm][fn][p * 8 + e]) - m0) - acc_read(zt[fm][fn][p * 8 + e]);
    slab_store16(rd, rowb ^ (((fm & 1) * 4 + p) << 4), (fm >> 1) * kImgBytesSlab + fn * 32 * kRowBytes, dd);
  };
  // The stores of D have little arithmetic of their own to hide behind, so column 0's second
  // pass is interleaved with column 1's first pass, whose exponentials cover them.
#pragma unroll
  for (int fm = 0; fm < 4; ++fm)
#pragma unroll
    for (int p = 0; p < 2; ++p) sums8(0, fm, p);
  float m0 = 0.f;
  if (WRITE_D) m0 = mean_of(0);
#pragma unroll
  for (int fm = 0; fm < 4; ++fm)
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      sums8(1, fm, p);
      if (WRITE_D) factor8(0, fm, p, m0);
    }
  if (WRITE_D) {
    m0 = mean_of(1);
#pragma unroll
    for (int fm = 0; fm < 4; ++fm)
#pragma unroll
      for (int p = 0; p < 2; ++p) factor8(1, fm, p, m0);
  }
#pragma unroll
  for (int fn = 0; fn < 2; ++fn) {
    sm.Z_s[fn] = Zs[fn]; sm.A_s[fn] = As[fn]; sm.Z_t[fn] = Zt[fn];
    if (DIAG) { sm.B_t[fn] = Bt[fn]; sm.cnt[fn] = cnt[fn]; }
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
        int v = v0 + entry_of_tile_row(r + 32 * i);   // staged row order, see entry_of_tile_row
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
                     wave * 64, v0, a.V, tail, lane, a.heavy, (int64_t)tt * kTileTokens + wave * 64);
  }
  if (!PASS2)
    write_partials(st, a.part, a.strips, strip, a.n_pad, (int64_t)tt * kTileTokens + wave * 64, lane);
}

// ---------------------------------------------------------------------------------------
// Logit passes, direct global->LDS staging.
//
// Same tile, MFMA roles and epilogues as logit_pass_kernel, but the k-tiles are moved by
// global_load_lds_dwordx4 (no register staging) into a three-stage LDS ring, two k-steps
// ahead of the MFMAs, from tile images that already have the LDS layout (row_image_kernel
// below): one wave instruction moves 1 KiB of consecutive bytes, lane l its 16 bytes at 16 l.
// The teacher and student k-loops form one pipeline of H_t/64 + H_s/64 steps per vocabulary
// tile.
//
// The loads are written as inline assembly (M0 = LDS destination of the wave, 64-bit scalar
// base + 32-bit lane offset within the block) and waited for with explicit
// s_waitcnt vmcnt(N): the loads return in order, so "at most the 12 loads of the next stage
// outstanding" means this stage has landed.  Compiler-issued loads in between only make the
// count larger, i.e. the wait longer.
// ---------------------------------------------------------------------------------------
constexpr int kDmaStages = 3;
constexpr int kDmaLds = kDmaStages * kLogitStage;           // 144 KiB
constexpr int kDmaPerWave = (kTileVocab + kTileTokens) / 8 / 4;   // 12 wave-loads per stage

// Row images.  The direct-to-LDS logit kernel reads all four operands as LDS images of its
// k-steps: [rows, H] row-major (optionally gathered through row_idx) is re-laid as tiles of
// `th` consecutive rows; block (tile, kt) holds their k-entries 64 kt .. 64 kt + 63, row r at
// r * 128 B, its 16-byte chunk c at chunk position c ^ ((r >> 1) & 7); rows >= n_rows are
// zero.  Blocks of one tile are consecutive in kt.  Every wave-load then moves 1 KiB of
// consecutive bytes and no operand needs 32-bit lane offsets from its base.  With `permute`
// (the W operands) tile row r holds source row entry_of_tile_row(r) of the tile.

__global__ __launch_bounds__(256) void row_image_kernel(RowImageArgs a) {
  const int kt = blockIdx.x;
  const int64_t tile = blockIdx.y;
  uint4* blk = a.img + ((tile * a.nk + kt) * a.th) * 8;
  for (int q = threadIdx.x; q < a.th * 8; q += 256) {
    const int r = q >> 3, pos = q & 7, c = pos ^ ((r >> 1) & 7);
    const int64_t row = tile * a.th + (a.permute ? entry_of_tile_row(r) : r);
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
// the B block; lane l moves bytes 16 l .. 16 l + 15 of that KiB.  lds_wave = the stage's LDS
// address + 1024 wave; voffw[j] = 16 lane + 1024 (wave + 4 j): the wave's part of both addresses
// is folded into operands that are set up once, the rest is a literal.
template <int I>
__device__ __forceinline__ void dma_one(uint32_t lds_wave, const uint32_t (&voffw)[8], const char* sA,
                                        const char* sB) {
  if constexpr (I < kTileVocab / 32)
    dma16_at<4 * I * 1024>(lds_wave, voffw[I], sA);
  else
    dma16_at<(kTileVocab / 8 + 4 * (I - kTileVocab / 32)) * 1024>(lds_wave, voffw[I - kTileVocab / 32], sB);
}

// One staged k-step (4 sub-steps of 8 MFMAs) of the 128 x 64 wave tile.  On entry fa[0],
// fb[0] hold the fragments of sub-step 0.  The instruction order is pinned: after each MFMA
// one or two side operations are issued in its shadow -- an LDS read of a fragment of the
// next sub-step (fragments are double-buffered), one of the 12 global->LDS loads of the
// stage two k-steps ahead (every k-step loads) or a piece of the pipeline's bookkeeping -- so
// that neither the LDS latency nor the vector-memory issue holds up the matrix pipe.  The one
// barrier of the k-step sits before the last sub-step: by then every fragment of this stage is
// in registers, and the last sub-step's MFMAs cover the reads of the next stage's first
// fragments (the following ring slot, whose loads were issued one k-step earlier and are waited
// for here).  LAST: no next stage in this vocabulary tile; no barrier and no fragment reads.
// FRESH: the k-step starts a new accumulation (first k-step of a head): its first MFMA on each
// block takes a zero addend, so the accumulators are never cleared.
// RELAXED > 0 (with `relaxed` set): the wait before the barrier lets RELAXED more operations
// stay in flight.  The counter takes loads and stores in the order of issue; the first k-step
// of a tile follows an epilogue that issued at least RELAXED stores after the loads this wait is
// for, and waiting for "all but this step's 9 loads" would mean waiting for every one of them.
// Ring and load state: r_rd = address (LDS base + 1024 wave + slot) of the slot consumed, on
// return that of the next k-step; swA/swB = the lane's fragment offsets from such an address
// per sub-step; (a_lo, a_hi), (b_lo, b_hi) = the blocks that the previous k-step loaded, on
// return those that this one loaded.
template <bool LAST, bool FRESH, int RELAXED>
__device__ __forceinline__ void sweep_kstep(f32x16 (&acc)[4][2], bf16x8 (&fa)[2][4], bf16x8 (&fb)[2][2],
                                            uint32_t& r_rd, uint32_t ring_begin, uint32_t ring_end,
                                            const uint32_t (&swA)[4], const uint32_t (&swB)[4],
                                            const uint32_t (&voffw)[8], uint32_t& a_lo, uint32_t& a_hi,
                                            uint32_t& b_lo, uint32_t& b_hi, bool relaxed = false) {
  static_assert(9 + RELAXED <= 63, "the wait count has six bits");
  const f32x16 kZeroTile = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  uint32_t r_nx, r_wr;
#define ADWIN_FENCE __builtin_amdgcn_sched_barrier(0);
#define ADWIN_RA(KK, I) fa[((KK) + 1) & 1][I] = lds_frag(xa)[(I) * 32 * kRowBytes / 16]; ADWIN_FENCE
#define ADWIN_RB(KK, I) fb[((KK) + 1) & 1][I] = lds_frag(xb)[(I) * 32 * kRowBytes / 16]; ADWIN_FENCE
#define ADWIN_MM(KK, FMI, FNI)                                                                  \
  acc[FMI][FNI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[(KK) & 1][FMI], fb[(KK) & 1][FNI], \
                                                          (FRESH && (KK) == 0) ? kZeroTile : acc[FMI][FNI], 0, 0, 0); \
  ADWIN_FENCE
#define ADWIN_DMA(I) dma_one<I>(r_wr, voffw, addr_of(a_lo, a_hi), addr_of(b_lo, b_hi)); ADWIN_FENCE
  // sub-step KK: 8 MFMAs; reads of the next sub-step's fragments from slot R when READ; H0..H3:
  // bookkeeping in the shadows of the first four MFMAs.  xa, xb: the lane's LDS addresses of its
  // first A and B fragment, formed once (and kept from being re-associated with the fragments'
  // constant offsets, which belong in the read instructions).
#define ADWIN_SUB(KK, READ, R, D0, D1, D2, H0, H1, H2, H3)                    \
  {                                                                     \
    uint32_t xa = 0, xb = 0;                                            \
    ADWIN_MM(KK, 0, 0)                                                  \
    if constexpr (READ) {                                               \
      xa = (R) + swA[((KK) + 1) & 3]; xb = (R) + swB[((KK) + 1) & 3];   \
      asm volatile("" : "+v"(xa), "+v"(xb));                            \
      ADWIN_RA(KK, 0)                                                   \
    }                                                                   \
    H0 ADWIN_FENCE                                                      \
    ADWIN_MM(KK, 0, 1) if constexpr (READ) { ADWIN_RB(KK, 0) } H1 ADWIN_FENCE \
    ADWIN_MM(KK, 1, 0) if constexpr (READ) { ADWIN_RA(KK, 1) } H2 ADWIN_FENCE \
    ADWIN_MM(KK, 1, 1) if constexpr (READ) { ADWIN_RB(KK, 1) } H3 ADWIN_FENCE \
    ADWIN_MM(KK, 2, 0) if constexpr (READ) { ADWIN_RA(KK, 2) }          \
    ADWIN_MM(KK, 2, 1) if constexpr (READ) { ADWIN_RA(KK, 3) } ADWIN_DMA(D0) \
    ADWIN_MM(KK, 3, 0) ADWIN_DMA(D1)                                    \
    ADWIN_MM(KK, 3, 1) ADWIN_DMA(D2)                                    \
  }
  ADWIN_FENCE
  ADWIN_SUB(0, true, r_rd, 0, 1, 2,
            { r_nx = ring_next<kLogitStage>(r_rd, ring_begin, ring_end); }, { r_wr = ring_next<kLogitStage>(r_nx, ring_begin, ring_end); },
            { addr_advance<kImgABytes>(a_lo, a_hi); }, { addr_advance<kImgBBytes>(b_lo, b_hi); })
  ADWIN_SUB(1, true, r_rd, 3, 4, 5, {}, {}, {}, {})
  ADWIN_SUB(2, true, r_rd, 6, 7, 8, {}, {}, {}, {})
  if constexpr (!LAST) {
    // loads issued after those of the next stage: the 9 above
    if constexpr (RELAXED > 0) {
      if (relaxed) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" :: "n"(9 + RELAXED) : "memory");
      else asm volatile("s_waitcnt vmcnt(9) lgkmcnt(0)" ::: "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(9) lgkmcnt(0)" ::: "memory");
    }
    __syncthreads();
  }
  ADWIN_FENCE
  ADWIN_SUB(3, !LAST, r_nx, 9, 10, 11, {}, {}, {}, {})
  r_rd = r_nx;
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

  uint32_t voffw[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    voffw[j] = (uint32_t)lane * 16u + (uint32_t)(wave + 4 * j) * 1024u;
    asm volatile("" : "+v"(voffw[j]));   // kept in registers, not recomputed at every load
  }
  // ring slot addresses carry the wave's KiB (for the loads); the fragment offsets take it out again
  const uint32_t ring_begin = lds0 + (uint32_t)wave * 1024u, ring_end = ring_begin + kDmaStages * kLogitStage;
  uint32_t swA[4], swB[4];
  {
    const int key = (lane >> 1) & 7, half = lane >> 5;
    const uint32_t rowoff = (uint32_t)(lane & 31) * kRowBytes - (uint32_t)wave * 1024u;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      swA[kk] = rowoff + (uint32_t)(((kk * 2 + half) ^ key) << 4);
      swB[kk] = swA[kk] + (uint32_t)(kTileVocab * kRowBytes + wave * 64 * kRowBytes);
    }
  }
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
  // before it is consumed, also across head and tile boundaries (the next tile's first two steps
  // are loaded during this tile's last two, i.e. before and under the epilogue).  ld*: the step
  // whose loads were issued last; past the strip's last step the walk wraps to the strip's first
  // tile, so that every k-step loads (those last blocks land in slots nobody reads any more).
  // (a, b) = the blocks of that step; a k-step moves them on by one block before it loads, so
  // at the start of a head they are set one block in front of it.
  uint32_t r_rd = ring_begin;  // ring slot (address) of the next step to consume
  int ld_vt = vt_begin, ld_k = 0, ld_lim = nk_t;
  bool ld_student = false;
  uint32_t a_lo, a_hi, b_lo, b_hi;
#define ADWIN_SET_BLOCKS(A, B)                                             \
  {                                                                        \
    const uint64_t pa = (uint64_t)(A) - kImgABytes, pb = (uint64_t)(B) - kImgBBytes; \
    a_lo = (uint32_t)pa; a_hi = (uint32_t)(pa >> 32);                      \
    b_lo = (uint32_t)pb; b_hi = (uint32_t)(pb >> 32);                      \
  }
#define ADWIN_COUNT_LOADS()                                                \
  {                                                                        \
    if (++ld_k == ld_lim) {                                                \
      ld_k = 0;                                                            \
      if (!ld_student) {                                                   \
        ld_student = true; ld_lim = nk_s;                                  \
        ADWIN_SET_BLOCKS(blocks_ws(ld_vt), sHs)                            \
      } else {                                                             \
        ld_student = false; ld_lim = nk_t;                                 \
        ld_vt = ld_vt + 1 < vt_end ? ld_vt + 1 : vt_begin;                 \
        ADWIN_SET_BLOCKS(blocks_wt(ld_vt), sHt)                            \
      }                                                                    \
    }                                                                      \
  }
  ADWIN_SET_BLOCKS(blocks_wt(vt_begin), sHt)
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const uint32_t dst = ring_begin + (uint32_t)i * kLogitStage;
    addr_advance<kImgABytes>(a_lo, a_hi);
    addr_advance<kImgBBytes>(b_lo, b_hi);
    const char* ldA = addr_of(a_lo, a_hi);
    const char* ldB = addr_of(b_lo, b_hi);
    dma_one<0>(dst, voffw, ldA, ldB); dma_one<1>(dst, voffw, ldA, ldB);
    dma_one<2>(dst, voffw, ldA, ldB); dma_one<3>(dst, voffw, ldA, ldB);
    dma_one<4>(dst, voffw, ldA, ldB); dma_one<5>(dst, voffw, ldA, ldB);
    dma_one<6>(dst, voffw, ldA, ldB); dma_one<7>(dst, voffw, ldA, ldB);
    dma_one<8>(dst, voffw, ldA, ldB); dma_one<9>(dst, voffw, ldA, ldB);
    dma_one<10>(dst, voffw, ldA, ldB); dma_one<11>(dst, voffw, ldA, ldB);
    ADWIN_COUNT_LOADS()
  }
  // 16-byte stores a wave issues per tile in its epilogue, at the least (see sweep_kstep, RELAXED)
  constexpr int kEpilogueStores = MODE == kModeDz ? 16 : (kWriteE2 && kSingle ? 16 : 0) + (kWriteD ? 16 : 0);
  f32x16 zt[4][2], zs[4][2];
  bf16x8 fa[2][4], fb[2][2];
  // one k-step: consume slot r_rd, prefetch fragments from the following slot, load into the one after
  auto step = [&](auto last_c, auto fresh_c, auto relaxed_c, f32x16 (&acc)[4][2], bool relaxed)
                  __attribute__((always_inline)) {
    constexpr bool kLast = decltype(last_c)::value, kFresh = decltype(fresh_c)::value;
    constexpr int kRelaxed = decltype(relaxed_c)::value;
    sweep_kstep<kLast, kFresh, kRelaxed>(acc, fa, fb, r_rd, ring_begin, ring_end, swA, swB, voffw,
                                         a_lo, a_hi, b_lo, b_hi, relaxed);
    ADWIN_COUNT_LOADS()
  };
  const std::true_type yes{};
  const std::false_type no{};
  const std::integral_constant<int, 0> strict{};
  const std::integral_constant<int, kEpilogueStores> after_epilogue{};
  for (int vt = vt_begin; vt < vt_end; ++vt) {
    const int v0 = vt * kTileVocab;
    // Step 0 of this tile has landed once at most the 12 loads of step 1 are outstanding.  For
    // the strip's first tile that is waited for here; for every later tile it was waited for
    // before the previous tile's epilogue (below): the counter takes loads and stores in order,
    // so a wait placed here would also wait for nearly all of that epilogue's stores.
    if (vt == vt_begin) wait_vm<kDmaPerWave>();
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[0][i] = lds_frag(r_rd + swA[0])[i * 32 * kRowBytes / 16];
#pragma unroll
    for (int i = 0; i < 2; ++i) fb[0][i] = lds_frag(r_rd + swB[0])[i * 32 * kRowBytes / 16];
    // teacher: nk_t k-steps (the first on a zero addend; after an epilogue its wait leaves that
    // epilogue's stores in flight), then student: nk_s k-steps, the last without a barrier
    step(no, yes, after_epilogue, zt, vt != vt_begin);
    for (int s = 1; s < nk_t; ++s) step(no, no, strict, zt, false);
    step(no, yes, strict, zs, false);
    for (int s = 1; s + 1 < nk_s; ++s) step(no, no, strict, zs, false);
    step(yes, no, strict, zs, false);
    wait_vm<kDmaPerWave>();                    // the next tile's step 0 (see the top of the loop)
    const bool tail = v0 + kTileVocab > a.V;
    if (MODE == kModeStats) {
      stats_epilogue(zs, zt, st, v0, a.V, tail, lane);
    } else {
      __bf16* blk = a.slab + ((int64_t)tt_local * (a.Vp / kBK) + 2 * vt) * kSlabBlock;
      float* m0t = a.mu0t ? a.mu0t + (int64_t)vt * a.mu0t_stride + (int64_t)tt_local * kTileTokens + wave * 64
                          : nullptr;
      if (MODE == kModeDz) {
        dz_epilogue(zs, zt, lse2, mu, blk, wave * 64, v0, a.V, tail, lane, a.heavy,
                    (int64_t)tt * kTileTokens + wave * 64);
      } else if (tail) {
        single_epilogue<true, kDiag, kWriteD, kWriteE2>(zs, zt, sm, rs2, rt2, mu, zyt, yid, blk, a.e2_off, wave * 64, v0, a.V, lane, m0t);
      } else {
        single_epilogue<false, kDiag, kWriteD, kWriteE2>(zs, zt, sm, rs2, rt2, mu, zyt, yid, blk, a.e2_off, wave * 64, v0, a.V, lane, m0t);
      }
    }
  }
#undef ADWIN_COUNT_LOADS
#undef ADWIN_SET_BLOCKS
  wait_vm<0>();      // the strip's last two k-steps loaded blocks nobody reads: landed before the LDS is released
  const int64_t row0 = (int64_t)tt * kTileTokens + wave * 64;
  if (MODE == kModeStats) write_partials(st, a.part, a.strips, strip, a.n_pad, row0, lane);
  else if (kSingle) write_sums<kDiag>(sm, a.part, a.strips, strip, a.n_pad, row0, lane);
}

// ---------------------------------------------------------------------------------------
// Merge of the strip partials, KL_t and c_t.  One wave per computed row.
// ---------------------------------------------------------------------------------------

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
  float kl = kl_from_sums(mu, ms - mt, Zs, Zt);
  // a row without a finite log-sum-exp, mean or KL is excluded: zeros in every output
  const bool dead = !(fabsf(lse_s) < 3.0e38f) || !(fabsf(lse_t) < 3.0e38f) || !(fabsf(kl) < 3.0e38f) ||
                    !(fabsf(mu) < 3.0e38f);
  if (dead) kl = 0.f;
  if (lane == 0) {
    a.lse2[r] = dead ? 0.f : lse_s * kLog2e;
    a.mu[r] = dead ? 0.f : mu;
    a.klr[r] = kl;
    a.lse_s[r] = dead ? 0.f : lse_s;
    a.alive[r] = dead ? 0.f : 1.f;
  }
  if (r >= a.n_rows) return;                // padding rows feed pass 2 only
  const int64_t t = a.row_idx[r];
  float c = 0.f;
  uint32_t flag = dead ? ADWIN_DEV_NONFINITE : 0u;
  if (a.ids && a.c && !dead) {
    const int y = a.ids[t];
    if (y >= 0 && y < a.V) {
      const float zy_s = dot_bf16_row(a.h_s + t * a.H_s, a.W_s + (int64_t)y * a.H_s, a.H_s, lane);
      const float zy_t = dot_bf16_row(a.h_t + t * a.H_t, a.W_t + (int64_t)y * a.H_t, a.H_t, lane);
      c = (zy_s - lse_s) - (zy_t - lse_t);
    } else {
      flag |= ADWIN_DEV_BAD_ID;
    }
  }
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
  float kl = kl_from_sums(mu, (b.ref_s2[r] - b.ref_t2[r]) * kLn2, Zs, Zt);
  const float iz = 1.f / Zs;
  float ent = lse_t - Bt / Zt;              // H[p_t] = lse_t - E_{p_t}[z_t]; both sums share the reference
  // a row without a finite log-sum-exp, mean or KL (logits beyond the range the fixed
  // references cover, or non-finite inputs) is excluded: zeros in every output
  const bool dead = !(fabsf(lse_s) < 3.0e38f) || !(fabsf(lse_t) < 3.0e38f) || !(fabsf(kl) < 3.0e38f) ||
                    !(fabsf(A) < 3.0e38f) || !(fabsf(mu) < 3.0e38f) || !(iz > 0.f) || !(iz < 3.0e38f) ||
                    (a.diag && !(fabsf(ent) < 3.0e38f));
  if (dead) { kl = 0.f; ent = 0.f; }
  if (lane == 0) {
    b.mu_out[r] = dead ? 0.f : mu;
    b.inv_z[r] = dead ? 0.f : iz;
    a.klr[r] = kl;
    a.lse_s[r] = dead ? 0.f : lse_s;
  }
  if (r >= a.n_rows) return;
  const int64_t t = a.row_idx[r];
  float c = 0.f, logp_t = 0.f;
  bool have_y = false;
  uint32_t flag = dead ? ADWIN_DEV_NONFINITE : 0u;
  if (a.ids && (a.c || a.t_logp || a.t_rank || a.cr) && !dead) {
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
  if (lane == 0) {
    if (flag && a.status) atomicOr(a.status, flag);
    if (a.kl) a.kl[t] = kl;
    if (a.c) a.c[t] = c;
    if (a.t_logp) a.t_logp[t] = logp_t;
    if (a.t_entropy) a.t_entropy[t] = ent;
    if (a.t_rank) a.t_rank[t] = have_y ? (int32_t)cnt + 1 : 0;
    if (a.cr) a.cr[r] = c;
  }
}

// Logits of the sampled token under both models, z_s[y_t] = h_s . W_s[y_t] and
// z_t[y_t] = h_t . W_t[y_t], and the token id (-1 when there is none or it is out of range),
// per computed row.  The references of the single sweep are built from them (make_refs_kernel)
// and the diagnostics sweep compares against z_t[y_t] to count the entries the teacher ranks
// above y_t (Sec. 3.1).  One wave per row.

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
// Launchers
// ---------------------------------------------------------------------------------------
hipError_t sweep_kernels_opt_in() {
  hipError_t e;
#define ADWIN_OPT_IN(KERNEL, BYTES)                                                              \
  e = hipFuncSetAttribute((const void*)KERNEL, hipFuncAttributeMaxDynamicSharedMemorySize, BYTES); \
  if (e != hipSuccess) return e;
  ADWIN_OPT_IN(logit_pass_kernel<false>, kLogitLds)
  ADWIN_OPT_IN(logit_pass_kernel<true>, kLogitLds)
  ADWIN_OPT_IN(logit_pass_dma_kernel<kModeStats>, kDmaLds)
  ADWIN_OPT_IN(logit_pass_dma_kernel<kModeDz>, kDmaLds)
  ADWIN_OPT_IN(logit_pass_dma_kernel<kModeSingle>, kDmaLds)
  ADWIN_OPT_IN(logit_pass_dma_kernel<kModeSingleDiag>, kDmaLds)
  ADWIN_OPT_IN(logit_pass_dma_kernel<kModeSingleE2>, kDmaLds)
  ADWIN_OPT_IN(logit_pass_dma_kernel<kModeSingleE2Diag>, kDmaLds)
  ADWIN_OPT_IN(logit_pass_dma_kernel<kModeSingleFwd>, kDmaLds)
  ADWIN_OPT_IN(logit_pass_dma_kernel<kModeSingleFwdDiag>, kDmaLds)
#undef ADWIN_OPT_IN
  return hipSuccess;
}

hipError_t launch_row_image(const RowImageArgs& a, unsigned tiles, hipStream_t st) {
  row_image_kernel<<<dim3((unsigned)a.nk, tiles), 256, 0, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_logit_pass(int mode, bool dma, const LogitPassArgs& a, unsigned grid, hipStream_t st) {
  if (!dma) {
    if (mode == kModeStats) logit_pass_kernel<false><<<grid, 256, kLogitLds, st>>>(a);
    else if (mode == kModeDz) logit_pass_kernel<true><<<grid, 256, kLogitLds, st>>>(a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
  }
  switch (mode) {
    case kModeStats: logit_pass_dma_kernel<kModeStats><<<grid, 256, kDmaLds, st>>>(a); break;
    case kModeDz: logit_pass_dma_kernel<kModeDz><<<grid, 256, kDmaLds, st>>>(a); break;
    case kModeSingle: logit_pass_dma_kernel<kModeSingle><<<grid, 256, kDmaLds, st>>>(a); break;
    case kModeSingleDiag: logit_pass_dma_kernel<kModeSingleDiag><<<grid, 256, kDmaLds, st>>>(a); break;
    case kModeSingleE2: logit_pass_dma_kernel<kModeSingleE2><<<grid, 256, kDmaLds, st>>>(a); break;
    case kModeSingleE2Diag: logit_pass_dma_kernel<kModeSingleE2Diag><<<grid, 256, kDmaLds, st>>>(a); break;
    case kModeSingleFwd: logit_pass_dma_kernel<kModeSingleFwd><<<grid, 256, kDmaLds, st>>>(a); break;
    case kModeSingleFwdDiag: logit_pass_dma_kernel<kModeSingleFwdDiag><<<grid, 256, kDmaLds, st>>>(a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_token_logit(const TokenLogitArgs& a, hipStream_t st) {
  token_logit_kernel<<<(unsigned)((a.n_pad + 3) / 4), 256, 0, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_make_refs(const float* part, int64_t n_pad, const float* zy_s, const float* zy_t,
                            const int32_t* yid, float* ref_s2, float* ref_t2, float* mu0, hipStream_t st) {
  make_refs_kernel<<<(unsigned)((n_pad + 255) / 256), 256, 0, st>>>(part, n_pad, zy_s, zy_t, yid, ref_s2,
                                                                    ref_t2, mu0);
  return hipGetLastError();
}

hipError_t launch_merge_stats(const MergeArgs& a, hipStream_t st) {
  merge_stats_kernel<<<(unsigned)((a.n_pad + 3) / 4), 256, 0, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_merge_single(const MergeSingleArgs& a, hipStream_t st) {
  merge_single_kernel<<<(unsigned)((a.rows + 3) / 4), 256, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace adwin
