// Driver for the host-sanitizer test: exercises the pure-host half of libadwin_opd (the planner
// of Sec. 4.1's integer bookkeeping, the plan blob, the scheduler and the staleness counters of
// Sec. 4.2 / 4.1) on seeded ragged batches, with every buffer sized exactly, so that an
// out-of-bounds access, a signed overflow or a misaligned store is reported by
// AddressSanitizer / UndefinedBehaviorSanitizer.  Built by tests/test_host_sanitizers.py with
// the host compiler only; no GPU code is involved.  Checks a few invariants itself; parity with
// the oracle is the business of tests/test_host_abi.py.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "host_plan.h"

namespace adwin {
const char* last_hip_error_text() { return ""; }   // the HIP-side state is not part of this build
}

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond);   \
      return 1;                                                            \
    }                                                                      \
  } while (0)

static int one_case(std::mt19937_64& g, int case_id) {
  const int32_t B = 1 + (int32_t)(g() % (case_id % 7 == 0 ? 3000 : 40));
  std::vector<int64_t> off((size_t)B + 1);
  std::vector<int32_t> win((size_t)B);
  off[0] = 0;
  for (int32_t i = 0; i < B; ++i) {
    int64_t len = (int64_t)(g() % 700);
    if (g() % 5 == 0) len = 0;
    if (case_id % 11 == 0 && i == 0) len = 200000;             // one long rollout
    off[i + 1] = off[i] + len;
    win[i] = (int32_t)(g() % 900);
    if (g() % 6 == 0) win[i] = 0;
    if (g() % 9 == 0) win[i] = INT32_MAX;                      // window far beyond the rollout
  }
  const int64_t T = off[B];
  std::vector<int32_t> n((size_t)B);
  int64_t n_adm = -1;
  CHECK(adwin_opd_plan_host(T, B, off.data(), win.data(), n.data(), nullptr, nullptr, &n_adm) == ADWIN_OK);
  int64_t sum = 0;
  for (int32_t i = 0; i < B; ++i) {
    const int64_t len = off[i + 1] - off[i];
    CHECK(n[i] == (win[i] < len ? win[i] : len));
    sum += n[i];
  }
  CHECK(sum == n_adm);
  std::vector<int64_t> rows((size_t)n_adm);                    // exactly N entries
  std::vector<int32_t> seq((size_t)n_adm);
  CHECK(adwin_opd_plan_host(T, B, off.data(), win.data(), n.data(), rows.data(), seq.data(), &n_adm) == ADWIN_OK);
  for (int64_t k = 0; k < n_adm; ++k) {
    CHECK(rows[k] >= off[seq[k]] && rows[k] < off[seq[k]] + n[seq[k]]);
    if (k) CHECK(rows[k] > rows[k - 1]);
  }
  for (int probe = 0; probe < 2; ++probe)
    for (int red = ADWIN_RED_SEQ_MEAN; red <= ADWIN_RED_TOKEN_MEAN; ++red) {
      std::vector<unsigned char> blob;
      const adwin::HostPlan hp = adwin::make_host_plan(T, B, off.data(), win.data(), probe, red, &blob);
      const adwin::PlanBlobLayout L(B);
      CHECK(blob.size() == L.bytes);
      CHECK(hp.n_adm == n_adm && hp.n_rows == (probe ? T : n_adm));
      CHECK(hp.n_pad % adwin::kTileTokens == 0 && hp.n_pad >= hp.n_rows && hp.n_pad < hp.n_rows + adwin::kTileTokens);
      const int64_t* comp = (const int64_t*)(blob.data() + L.o_comp_off);
      const int32_t* chunk = (const int32_t*)(blob.data() + L.o_chunk_off);
      const float* ap = (const float*)(blob.data() + L.o_alpha_p);
      CHECK(comp[0] == 0 && comp[B] == hp.n_rows && chunk[0] == 0 && chunk[B] == hp.n_chunks);
      for (int32_t i = 0; i < B; ++i) {
        const int64_t hi = probe ? off[i + 1] - off[i] : n[i];
        CHECK(comp[i + 1] - comp[i] == hi);
        CHECK(chunk[i + 1] - chunk[i] == (hi + adwin::kChunkRows - 1) / adwin::kChunkRows);
        CHECK(std::isfinite(ap[i]) && ap[i] >= 0.f);
      }
      const adwin::HostPlan counts = adwin::make_host_plan(T, B, off.data(), win.data(), probe, red, nullptr);
      CHECK(counts.n_rows == hp.n_rows && counts.n_chunks == hp.n_chunks);
    }
  // error paths leave the outputs alone
  if (B > 1 && off[B] > off[0]) {
    std::vector<int64_t> bad(off);
    bad[B] += 1;
    CHECK(adwin_opd_plan_host(T, B, bad.data(), win.data(), n.data(), nullptr, nullptr, &n_adm) == ADWIN_E_OFFSETS);
    std::vector<int32_t> neg(win);
    neg[B - 1] = -1;
    CHECK(adwin_opd_plan_host(T, B, off.data(), neg.data(), n.data(), nullptr, nullptr, &n_adm) == ADWIN_E_WINDOW);
  }
  // scheduler and staleness counters
  const int32_t K = 1 + (int32_t)(g() % ADWIN_MAX_CANDIDATES);
  std::vector<float> rho((size_t)K), snr((size_t)K);
  std::vector<int32_t> cand((size_t)K);
  for (int32_t k = 0; k < K; ++k) {
    rho[k] = (float)((double)(g() % 2001) / 1000.0 - 1.0);
    cand[k] = 1 + (int32_t)(g() % 4096);
  }
  CHECK(adwin_opd_snr(rho.data(), K, snr.data()) == ADWIN_OK);
  int32_t next = 0;
  CHECK(adwin_opd_next_window(rho.data(), cand.data(), K, 0.f, &next) == ADWIN_OK);
  bool member = false;
  for (int32_t k = 0; k < K; ++k) member = member || cand[k] == next;
  CHECK(member);
  const int32_t P = (int32_t)(g() % 50);
  std::vector<int32_t> age((size_t)P, 0);
  std::vector<uint8_t> pend((size_t)P), force((size_t)P);
  for (int32_t i = 0; i < P; ++i) { pend[i] = (uint8_t)(g() & 1); age[i] = (g() % 13 == 0) ? INT32_MAX : (int32_t)(g() % 7); }
  int32_t forced = -1;
  CHECK(adwin_opd_probe_staleness(age.data(), pend.data(), P, 5, force.data(), &forced) == ADWIN_OK);
  CHECK(forced >= 0 && forced <= P);
  return 0;
}

int main(int argc, char** argv) {
  const int cases = argc > 1 ? atoi(argv[1]) : 200;
  std::mt19937_64 g(20260528);
  for (int c = 0; c < cases; ++c)
    if (one_case(g, c)) return 1;
  // limits of the shape checks
  int64_t off2[2] = {0, (int64_t)1 << 31};
  int32_t w1[1] = {3}, n1[1];
  int64_t na = 0;
  if (adwin_opd_plan_host(off2[1], 1, off2, w1, n1, nullptr, nullptr, &na) != ADWIN_E_SHAPE) return 1;
  if (adwin_opd_plan_host(0, 0, off2, w1, n1, nullptr, nullptr, &na) != ADWIN_E_SHAPE) return 1;
  if (adwin_opd_strerror(ADWIN_E_MODE)[0] == 0 || adwin_opd_version() < 100) return 1;
  printf("ok %d cases\n", cases);
  return 0;
}
