// Fused path, host side: argument checks, workspace layout and the sequence of launches
// that makes one call (Sec. 4.1: supervision on the admitted prefix; Sec. 4.2: the probe
// audit against the full-rollout gradient).  The kernels are in sweep_kernels.hip,
// grad_kernels.hip and reduce_kernels.hip; nothing here touches device memory itself.
#include <optional>
#include <utility>
#include <vector>

#include "fused_shared.h"

namespace adwin {

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
      o_pp, o_pf, o_up, o_uf, o_seg, o_racc, o_uc, o_cacc, o_cS, o_cr, o_zy_s, o_zy_t, o_yid, o_dzT_p, o_dzT_f, o_hsT, o_summ, o_cosp,
      o_lse_s, o_heavy_cnt, o_heavy_v, total;
};

// Which kernels a scheme selects for this shape: the direct-to-LDS logit kernel pipelines at
// least two k-steps per head, so it needs both hidden sizes >= 128.  False: the scheme is not
// available for the shape.
static bool resolve_scheme(const adwin_opd_problem* p, bool* use_dma, bool* single) {
  const bool dma_ok = p->H_s >= 2 * kBK && p->H_t >= 2 * kBK;
  switch (p->scheme) {
    case ADWIN_SCHEME_AUTO: *use_dma = dma_ok; *single = dma_ok; return true;
    case ADWIN_SCHEME_SINGLE: *use_dma = true; *single = true; return dma_ok;
    case ADWIN_SCHEME_TWO_SWEEP: *use_dma = dma_ok; *single = false; return true;
    case ADWIN_SCHEME_TWO_SWEEP_REG: *use_dma = false; *single = false; return true;
    default: *use_dma = false; *single = false; return false;
  }
}

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
  (void)resolve_scheme(p, &L.use_dma, &L.single);     // validity was checked with the problem
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
  L.o_lse_s = take(sizeof(float) * (size_t)n_pad);
  L.o_heavy_cnt = take(sizeof(int32_t) * (size_t)n_pad);
  L.o_heavy_v = take(need_g ? sizeof(int32_t) * (size_t)kHeavySlots * (size_t)n_pad : 0);
  L.total = o;
  return L;
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
  {
    bool use_dma, single;
    if (!resolve_scheme(p, &use_dma, &single)) return ADWIN_E_MODE;
  }
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
  hipError_t e = sweep_kernels_opt_in();
  if (e != hipSuccess) return e;
  return grad_kernels_opt_in();
}

}  // namespace adwin

using namespace adwin;

extern "C" int adwin_opd_init(void) {
  ADWIN_HIP_TRY(sweep_kernels_opt_in());
  ADWIN_HIP_TRY(grad_kernels_opt_in());
  ADWIN_HIP_TRY(logits_kernels_opt_in());
  ADWIN_HIP_TRY(logits_static_setup());
  (void)first_use_on_device(0);      // the calls need not repeat it on this device
  (void)first_use_on_device(1);
  return ADWIN_OK;
}

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

  // one timed span at a time: starting a phase ends the previous one (no-ops without a timer)
  std::optional<PhaseScope> scope;
  auto phase = [&](int ph) { scope.reset(); scope.emplace(timer, ph); };
  phase(ADWIN_PHASE_SETUP);
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

  HeavyList heavy;
  heavy.cnt = (int32_t*)(ws + L.o_heavy_cnt); heavy.v = (int32_t*)(ws + L.o_heavy_v);
  if (hp.n_rows > 0) {
    ADWIN_HIP_TRY(launch_build_rows(pl, p->B, hp.n_rows, n_pad, stream));
    ADWIN_HIP_TRY(launch_fill_u32((uint32_t*)heavy.cnt, n_pad, 0u, stream));
    const int vt_total = (int)(L.Vp / kTileVocab);
    const int n_tiles = (int)(n_pad / kTileTokens);
    // tile images of W_s^T for the gradient GEMM
    const int h_tiles = (p->H_s + kGradTile - 1) / kGradTile;
    if (need_g) {
      ADWIN_HIP_TRY(launch_wst_image(p->W_s, ws + L.o_WsT, p->V, p->H_s, (int)(L.Vp / kBK), h_tiles, stream));
    }
    const bool use_dma = L.use_dma;
    if (use_dma) {
      // tile images of the logit operands: vocabulary tiles of 128 rows (zero beyond V),
      // token tiles of 256 computed rows gathered through row_idx
      RowImageArgs ia;
      ia.row_idx = nullptr; ia.n_rows = p->V; ia.th = kTileVocab; ia.permute = 1;
      ia.src = (const uint4*)p->W_t; ia.img = (uint4*)(ws + L.o_wt_img); ia.H = p->H_t; ia.nk = p->H_t / kBK;
      ADWIN_HIP_TRY(launch_row_image(ia, (unsigned)vt_total, stream));
      ia.src = (const uint4*)p->W_s; ia.img = (uint4*)(ws + L.o_ws_img); ia.H = p->H_s; ia.nk = p->H_s / kBK;
      ADWIN_HIP_TRY(launch_row_image(ia, (unsigned)vt_total, stream));
      ia.row_idx = pl.row_idx; ia.n_rows = n_pad; ia.th = kTileTokens; ia.permute = 0;
      ia.src = (const uint4*)p->h_t; ia.img = (uint4*)(ws + L.o_ht_img); ia.H = p->H_t; ia.nk = p->H_t / kBK;
      ADWIN_HIP_TRY(launch_row_image(ia, (unsigned)n_tiles, stream));
      ia.src = (const uint4*)p->h_s; ia.img = (uint4*)(ws + L.o_hs_img); ia.H = p->H_s; ia.nk = p->H_s / kBK;
      ADWIN_HIP_TRY(launch_row_image(ia, (unsigned)n_tiles, stream));
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
    la.tg = env_int("ADWIN_TG", 4);      // tuning override
    la.Wt_img = (const char*)(ws + L.o_wt_img); la.Ws_img = (const char*)(ws + L.o_ws_img);
    la.ht_img = (const char*)(ws + L.o_ht_img); la.hs_img = (const char*)(ws + L.o_hs_img);
    la.heavy = heavy;
    MergeArgs m;
    m.part = la.part; m.strips = L.strips; m.n_pad = n_pad; m.n_rows = hp.n_rows;
    m.row_idx = pl.row_idx;
    m.h_s = la.h_s; m.h_t = la.h_t; m.W_s = la.W_s; m.W_t = la.W_t;
    m.H_s = p->H_s; m.H_t = p->H_t; m.V = p->V; m.ids = p->ids;
    m.lse2 = (float*)(ws + L.o_lse2); m.mu = (float*)(ws + L.o_mu); m.klr = klr;
    m.lse_s = (float*)(ws + L.o_lse_s); m.alive = (float*)(ws + L.o_invz);
    m.kl = p->kl; m.c = p->c; m.status = p->status_dev;
    m.diag = diag ? 1 : 0; m.t_logp = p->t_logp; m.t_entropy = p->t_entropy; m.t_rank = p->t_rank;
    m.cr = sampled ? (float*)(ws + L.o_cr) : nullptr;
    GradArgs ga;
    ga.slab = la.slab; ga.WsT = (const __bf16*)(ws + L.o_WsT); ga.nk_total = (int)(L.Vp / kBK);
    ga.g = gws; ga.H = p->H_s; ga.h_tiles = h_tiles; ga.ksplit = L.ksplit;
    ga.out_rows = (int64_t)1 << 62; ga.accumulate = 0;
    if (L.single) {
      // Single sweep.  (1) online statistics of vocabulary tile 0 and the sampled token's
      // logits give each row its fixed references; (2) per row slab: one sweep over the
      // vocabulary producing the strip sums and the gradient factors, the merge of the
      // slab's rows, the combine pass over the factors and the GEMM of dz with W_s.
      la.tile0 = 0; la.n_tiles = n_tiles; la.strips = 1; la.vt_total = 1;
      {
        const int groups = (n_tiles + la.tg - 1) / la.tg;
        ADWIN_HIP_TRY(launch_logit_pass(kModeStats, true, la, (unsigned)(groups * la.tg), stream));
        if (p->ids || diag) {      // without ids: id -1 on every row, which the diagnostics sweep expects
          TokenLogitArgs ta;
          ta.row_idx = pl.row_idx; ta.ids = p->ids;
          ta.h_s = la.h_s; ta.W_s = la.W_s; ta.h_t = la.h_t; ta.W_t = la.W_t;
          ta.H_s = p->H_s; ta.H_t = p->H_t; ta.V = p->V; ta.n_pad = n_pad;
          ta.zy_s = (float*)(ws + L.o_zy_s); ta.zy_t = (float*)(ws + L.o_zy_t);
          ta.yid = (int32_t*)(ws + L.o_yid);
          ADWIN_HIP_TRY(launch_token_logit(ta, stream));
        }
        ADWIN_HIP_TRY(launch_make_refs(la.part, n_pad, (const float*)(ws + L.o_zy_s),
                                       (const float*)(ws + L.o_zy_t),
                                       p->ids ? (const int32_t*)(ws + L.o_yid) : nullptr,
                                       (float*)(ws + L.o_lse2), (float*)(ws + L.o_ref_t2),
                                       (float*)(ws + L.o_mu), stream));
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
        const int sweep_mode = !need_g ? (diag ? kModeSingleFwdDiag : kModeSingleFwd)
                               : sampled ? (diag ? kModeSingleE2Diag : kModeSingleE2)
                                         : (diag ? kModeSingleDiag : kModeSingle);
        ADWIN_HIP_TRY(launch_logit_pass(sweep_mode, true, la, sweep_grid, stream));
        // this slab's rows are complete: KL_t, c_t, mu; then the logit gradient proper
        phase(ADWIN_PHASE_MERGE);
        MergeSingleArgs ms;
        ms.m = m; ms.m.strips = L.strips1;
        ms.ref_s2 = la.ref_s2; ms.ref_t2 = la.ref_t2;
        ms.mu_out = (float*)(ws + L.o_delta); ms.inv_z = (float*)(ws + L.o_invz);
        ms.row0 = r0; ms.rows = rows;
        ADWIN_HIP_TRY(launch_merge_single(ms, stream));
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
        ca.heavy = heavy;
        if (sampled) {       // contract the E2 factor; c_t and W_s[y_t] enter in finalize_kernel
          ga.slab = la.slab + la.e2_off;
          ga.half_tiles = 0;                       // output rows in the second half of g
          if (head) {        // the transposed operand of the head-weight GEMMs; the slab stays as it is
            phase(ADWIN_PHASE_DZ);
            ADWIN_HIP_TRY(launch_combine(true, true, ca, ga.row_tiles, stream));
          }
        } else {
          phase(ADWIN_PHASE_DZ);
          ADWIN_HIP_TRY(launch_combine(head, false, ca, ga.row_tiles, stream));
          ga.half_tiles = ga.row_tiles;            // output rows in the first half of g
        }
        phase(ADWIN_PHASE_GRAD);
        ADWIN_HIP_TRY(launch_grad_gemm(ga, stream));
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
          ha.alive = (const float*)(ws + L.o_invz);
          ADWIN_HIP_TRY(launch_hst_image(ha, h_tiles, stream));
          for (int which = 0; which < 2; ++which) {
            float* out = which == 0 ? p->dW_prefix : p->dW_full;
            if (!out) continue;
            wa.slab = (const __bf16*)(ws + (which == 0 ? L.o_dzT_p : L.o_dzT_f));
            wa.g = out;
            ADWIN_HIP_TRY(launch_grad_gemm(wa, stream));
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
        ADWIN_HIP_TRY(launch_logit_pass(kModeStats, use_dma, la, (unsigned)(groups * la.tg * L.strips), stream));
      }
      phase(ADWIN_PHASE_MERGE);
      ADWIN_HIP_TRY(launch_merge_stats(m, stream));
      const int strips2 = L.strips1;
      ga.g_rows = n_pad; ga.half_off = 0;
      for (int64_t r0 = 0; r0 < n_pad; r0 += L.slab_rows) {
        const int64_t rows = (n_pad - r0 < L.slab_rows) ? n_pad - r0 : L.slab_rows;
        la.tile0 = (int)(r0 / kTileTokens); la.n_tiles = (int)(rows / kTileTokens);
        la.strips = strips2;
        const int groups = (la.n_tiles + la.tg - 1) / la.tg;
        phase(ADWIN_PHASE_DZ);
        ADWIN_HIP_TRY(launch_logit_pass(kModeDz, use_dma, la, (unsigned)(groups * la.tg * strips2), stream));
        phase(ADWIN_PHASE_GRAD);
        ga.slab_row0 = r0;
        ga.row_tiles = (int)(rows / kGradTile); ga.half_tiles = ga.row_tiles;
        ADWIN_HIP_TRY(launch_grad_gemm(ga, stream));
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
    f.inv_z = (const float*)(ws + L.o_invz);
    // the fp32 part of g; the sampled estimator contracts E2 as stored and lists nothing
    f.heavy = heavy;
    if (p->estimator == ADWIN_EST_SAMPLED) f.heavy.cnt = nullptr;
    f.lse_s = (const float*)(ws + L.o_lse_s);
    f.mu = (const float*)(ws + (L.single ? L.o_delta : L.o_mu));
    f.h_s = (const __bf16*)p->h_s; f.h_t = (const __bf16*)p->h_t; f.W_t = (const __bf16*)p->W_t; f.H_t = p->H_t;
    f.cr = (L.single && p->estimator == ADWIN_EST_SAMPLED) ? (const float*)(ws + L.o_cr) : nullptr;
    f.ids = p->ids; f.W_s = (const __bf16*)p->W_s; f.V = p->V;
    f.grad_scale = p->grad_scale; f.dh_bf16 = p->dh_dtype == ADWIN_DT_BF16;
    f.dh_prefix = p->dh_prefix; f.dh_full = p->dh_full; f.rownorm = rownorm;
    ADWIN_HIP_TRY(launch_finalize(f, stream));
  }
  ADWIN_HIP_TRY(launch_segment_sums(pl, p->B, probe, klr, need_g ? rownorm : nullptr, seg, p->loss_prefix,
                                    p->loss_full, stream));
  PoolArgs pa;
  pa.pl = pl; pa.B = p->B; pa.probe = probe; pa.H = p->H_s; pa.g = gws;
  pa.pp = (float*)(ws + L.o_pp); pa.pf = (float*)(ws + L.o_pf);
  pa.up = (float*)(ws + L.o_up); pa.uf = (float*)(ws + L.o_uf);
  if (probe && need_g) {
    if (hp.n_chunks > 0) ADWIN_HIP_TRY(launch_pool_partial(pa, (int)hp.n_chunks, stream));
    ADWIN_HIP_TRY(launch_pool_final(pa, stream));
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
