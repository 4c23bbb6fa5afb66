// Host-side integer bookkeeping (Sec. 4.1: rollouts truncated at the window), the scheduler
// of Sec. 4.2, status strings and the version.  Nothing here touches the GPU or includes a HIP
// header: this file also builds with the host compiler alone (the sanitizer test does that).
#include <cmath>
#include <climits>
#include <cstring>

#include "host_plan.h"

namespace adwin {

int validate_ragged(int64_t T, int32_t B, const int64_t* offsets, const int32_t* window) {
  if (!offsets || !window) return ADWIN_E_NULL;
  if (B < 1 || T < 0 || T >= (int64_t(1) << 31)) return ADWIN_E_SHAPE;
  if (offsets[0] != 0) return ADWIN_E_OFFSETS;
  for (int32_t i = 0; i < B; ++i)
    if (offsets[i + 1] < offsets[i]) return ADWIN_E_OFFSETS;
  if (offsets[B] != T) return ADWIN_E_OFFSETS;
  for (int32_t i = 0; i < B; ++i)
    if (window[i] < 0) return ADWIN_E_WINDOW;
  return ADWIN_OK;
}

HostPlan make_host_plan(int64_t T, int32_t B, const int64_t* offsets, const int32_t* window,
                        int probe, int reduction, std::vector<unsigned char>* blob) {
  HostPlan hp;
  hp.T = T;
  hp.B = B;
  PlanBlobLayout L(B);
  unsigned char* base = nullptr;
  if (blob) {
    blob->assign(L.bytes, 0);
    base = blob->data();
  }
  int64_t n_adm = 0;
  for (int32_t i = 0; i < B; ++i) {
    const int64_t len = offsets[i + 1] - offsets[i];
    n_adm += window[i] < len ? (int64_t)window[i] : len;
  }
  int64_t comp = 0;
  int64_t chunks = 0;
  for (int32_t i = 0; i < B; ++i) {
    const int64_t len = offsets[i + 1] - offsets[i];
    const int64_t ni = window[i] < len ? (int64_t)window[i] : len;
    const int64_t hi = probe ? len : ni;
    if (base) {
      ((int64_t*)(base + L.o_offsets))[i] = offsets[i];
      ((int64_t*)(base + L.o_comp_off))[i] = comp;
      ((int32_t*)(base + L.o_n))[i] = (int32_t)ni;
      ((int32_t*)(base + L.o_chunk_off))[i] = (int32_t)chunks;
      double ap = 0.0, af = 0.0;
      if (reduction == ADWIN_RED_SEQ_MEAN) {
        ap = ni > 0 ? 1.0 / ((double)B * (double)ni) : 0.0;
        af = len > 0 ? 1.0 / ((double)B * (double)len) : 0.0;
      } else if (reduction == ADWIN_RED_SUM) {
        ap = af = 1.0;
      } else {
        ap = n_adm > 0 ? 1.0 / (double)n_adm : 0.0;
        af = T > 0 ? 1.0 / (double)T : 0.0;
      }
      ((float*)(base + L.o_alpha_p))[i] = (float)ap;
      ((float*)(base + L.o_alpha_f))[i] = (float)af;
    }
    comp += hi;
    chunks += (hi + kChunkRows - 1) / kChunkRows;
  }
  if (base) {
    ((int64_t*)(base + L.o_offsets))[B] = offsets[B];
    ((int64_t*)(base + L.o_comp_off))[B] = comp;
    ((int32_t*)(base + L.o_chunk_off))[B] = (int32_t)chunks;
  }
  hp.n_adm = n_adm;
  hp.n_rows = comp;
  hp.n_pad = (int64_t)align_up((size_t)comp, kTileTokens);
  hp.n_chunks = chunks;
  return hp;
}

}  // namespace adwin

extern "C" {

int adwin_opd_version(void) { return 100; }  // 0.1.0

const char* adwin_opd_strerror(int status) {
  switch (status) {
    case ADWIN_OK: return "ok";
    case ADWIN_E_NULL: return "a required pointer is NULL";
    case ADWIN_E_SHAPE:
      return "bad shape: need B>=1, 0<=T<2^31, V a positive multiple of 8, H_s and H_t positive "
             "multiples of 64";
    case ADWIN_E_OFFSETS: return "offsets must start at 0, be non-decreasing and end at T";
    case ADWIN_E_WINDOW: return "window lengths must be >= 0";
    case ADWIN_E_ALIGN: return "device pointers must be 16-byte aligned";
    case ADWIN_E_WORKSPACE: return "workspace is NULL, not 256-byte aligned or too small";
    case ADWIN_E_MODE:
      return "unknown mode, reduction, dh_dtype, estimator or scheme, struct_bytes mismatch, or an "
             "option the selected scheme does not offer";
    case ADWIN_E_HIP: {
      const char* t = adwin::last_hip_error_text();
      return t[0] ? t : "a HIP call failed";
    }
    default: return "unknown status";
  }
}

int adwin_opd_plan_host(int64_t T, int32_t B, const int64_t* offsets, const int32_t* window,
                        int32_t* n, int64_t* row_list, int32_t* row_seq, int64_t* n_adm) {
  int st = adwin::validate_ragged(T, B, offsets, window);
  if (st != ADWIN_OK) return st;
  if (!n || !n_adm) return ADWIN_E_NULL;
  int64_t total = 0;
  for (int32_t i = 0; i < B; ++i) {
    const int64_t len = offsets[i + 1] - offsets[i];
    const int64_t ni = window[i] < len ? (int64_t)window[i] : len;
    n[i] = (int32_t)ni;
    for (int64_t j = 0; j < ni; ++j) {
      if (row_list) row_list[total + j] = offsets[i] + j;
      if (row_seq) row_seq[total + j] = i;
    }
    total += ni;
  }
  *n_adm = total;
  return ADWIN_OK;
}

// Eq. 10: SNR(L) = rho^2 / (1 - rho^2).
int adwin_opd_snr(const float* rho, int32_t k, float* snr) {
  if (!rho || !snr) return ADWIN_E_NULL;
  if (k < 0) return ADWIN_E_SHAPE;
  for (int32_t i = 0; i < k; ++i) {
    const double r2 = (double)rho[i] * (double)rho[i];
    snr[i] = r2 >= 1.0 ? INFINITY : (float)(r2 / (1.0 - r2));
  }
  return ADWIN_OK;
}

// Sec. 4.2: L_{t+1} = min{L in the candidate list : rho_t(L) >= rho*}.
int adwin_opd_next_window(const float* rho, const int32_t* candidates, int32_t k, float rho_star,
                          int32_t* next) {
  if (!rho || !candidates || !next) return ADWIN_E_NULL;
  if (k < 1) return ADWIN_E_SHAPE;
  for (int32_t i = 0; i < k; ++i)
    if (candidates[i] <= 0) return ADWIN_E_WINDOW;
  const double thr = rho_star > 0.f ? (double)rho_star : std::sqrt(2.0) / 2.0;
  int32_t best = 0, longest = candidates[0];
  for (int32_t i = 0; i < k; ++i) {
    if (candidates[i] > longest) longest = candidates[i];
    if ((double)rho[i] >= thr && (best == 0 || candidates[i] < best)) best = candidates[i];
  }
  *next = best > 0 ? best : longest;
  return ADWIN_OK;
}

// Sec. 4.1: a probe older than the staleness limit is forced to complete.
int adwin_opd_probe_staleness(int32_t* age, const uint8_t* pending, int32_t n_probes, int32_t limit,
                              uint8_t* force, int32_t* n_forced) {
  if (n_probes < 0 || limit < 1) return ADWIN_E_SHAPE;
  if (n_probes > 0 && (!age || !pending || !force)) return ADWIN_E_NULL;
  int32_t cnt = 0;
  for (int32_t i = 0; i < n_probes; ++i) {
    if (pending[i]) {
      if (age[i] < INT32_MAX) age[i] += 1;
      force[i] = age[i] >= limit ? 1 : 0;
    } else {
      age[i] = 0;
      force[i] = 0;
    }
    cnt += force[i];
  }
  if (n_forced) *n_forced = cnt;
  return ADWIN_OK;
}

}  // extern "C"
