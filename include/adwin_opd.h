/*
 * libadwin_opd -- teacher-anchored per-token supervision for on-policy distillation
 * over ragged student rollouts, for one AMD MI355X (gfx950).
 *
 * What is computed (paper: ADWIN, "Adaptive Windows for Horizon-Aware On-Policy
 * Distillation"):
 *   - Sec. 4.1, synchronous path: the OPD loss is evaluated only on the first
 *     n_i = min(window_i, len_i) response positions of rollout i.
 *   - Eq. 2 at token level: KL_t = KL(softmax(W_s h_s[t]) || softmax(W_t h_t[t])),
 *     student first, teacher frozen, temperature 1 (App. B.1, OPD table).
 *   - Sec. 2.3 / App. A.1: sampled step cost c_t = log p_s(y_t) - log p_t(y_t).
 *   - Eq. 4 in expectation over y_t ~ p_s (equivalently dKL_t/dz_s with the teacher
 *     constant, App. A.1): dz_t = p_s * ((z_s - z_t) - E_{p_s}[z_s - z_t]);
 *     g_t = dz_t W_s is the gradient with respect to the student hidden state.
 *   - Sec. 4.2: alignment rho = cos(prefix-window gradient, full-rollout gradient),
 *     per rollout and after batch aggregation (Fig. 5: "macro" and "micro").
 *
 * Conventions common to every entry point
 *   - extern "C"; every function returns an int status: 0 = ADWIN_OK, negative =
 *     error.  Nothing throws, aborts or exits.  On an argument error no output
 *     buffer is touched and nothing is enqueued.
 *   - "host" pointers are ordinary CPU memory (pageable is fine) read synchronously
 *     during the call and free to be reused once it returns: what the device needs
 *     of them travels in kernel arguments, not in asynchronous copies;
 *     "device" pointers are HIP device memory on the current device, owned by the
 *     caller, row-major and contiguous, 16-byte aligned.
 *   - The library allocates no device memory.  All scratch comes from the caller's
 *     workspace (size from *_workspace_bytes); the one exception is
 *     adwin_opd_from_logits_static, whose scratch is a fixed array inside the library.
 *     What the library remembers between calls: per device, that the kernel attributes
 *     have been set (first call or adwin_opd_init) and the address of that array; per
 *     thread, the text of the last HIP error for adwin_opd_strerror.  No result of one
 *     call depends on an earlier one.
 *   - Work is enqueued on the caller's HIP stream (`hip_stream` is a hipStream_t, NULL
 *     = default stream) and the call returns without synchronising.  Outputs are
 *     defined once the stream has drained and the status was ADWIN_OK.  After a first
 *     call on the device or adwin_opd_init (either sets the kernel attributes) a call is
 *     nothing but kernel launches, so it may be captured in a HIP graph; the host arrays are read at
 *     capture, the device buffers at every replay.
 *   - Row t of the packed [T, .] arrays holds the hidden state (or logits) of the
 *     context (x, y_<t) and ids[t] = y_t: the caller has already applied the
 *     next-token shift and dropped prompt positions.
 *   - Results are deterministic, bit for bit from call to call: every sum is taken in
 *     a fixed order (where the head-weight gradient adds one slab's contribution to
 *     the previous ones with the hardware's floating-point add, each element is added
 *     to by exactly one lane per launch and the launches are ordered on the stream).
 */
#ifndef ADWIN_OPD_H
#define ADWIN_OPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define ADWIN_OK            0
#define ADWIN_E_NULL       -1  /* a required pointer is NULL                                  */
#define ADWIN_E_SHAPE      -2  /* T,B,V,H out of range: see adwin_opd_problem                  */
#define ADWIN_E_OFFSETS    -3  /* offsets[0]!=0, decreasing, or offsets[B]!=T                   */
#define ADWIN_E_WINDOW     -4  /* a window is negative                                         */
#define ADWIN_E_ALIGN      -5  /* a device pointer is not 16-byte aligned                      */
#define ADWIN_E_WORKSPACE  -6  /* workspace NULL, misaligned (256 B) or too small              */
#define ADWIN_E_MODE       -7  /* unknown mode / reduction / dh_dtype / estimator / scheme,    */
                               /* struct_bytes mismatch, or an option the selected scheme does */
                               /* not offer                                                    */
#define ADWIN_E_HIP        -8  /* a HIP call or kernel launch failed                           */

/* mode */
#define ADWIN_PREFIX_ONLY      0  /* compute the admitted rows only                            */
#define ADWIN_PREFIX_AND_FULL  1  /* probe audit: compute every row, both losses, alignment    */

/* reduction: weight alpha of one token's KL in the batch objective                            */
#define ADWIN_RED_SEQ_MEAN     0  /* alpha^p_i = 1/(B n_i),  alpha^f_i = 1/(B len_i)  (default) */
#define ADWIN_RED_SUM          1  /* alpha = 1                                                 */
#define ADWIN_RED_TOKEN_MEAN   2  /* alpha^p = 1/N_adm,      alpha^f = 1/T                     */

/* estimator: which per-token gradient dh / dz carries
 *   EXPECTED  p_s (Delta - KL_t): the gradient of the full-vocabulary KL_t, i.e. Eq. 4's
 *             per-token term in expectation over y_t ~ p_s (default)
 *   SAMPLED   c_t (e_{y_t} - p_s): Eq. 4's per-token term itself on the sampled token, c_t held
 *             constant; needs ids (rows with an id outside [0, V) get a zero gradient).  On
 *             the fused path it needs one gradient contraction instead of two.
 * KL_t, c_t, the window losses and every other output are the same under both. */
#define ADWIN_EST_EXPECTED  0
#define ADWIN_EST_SAMPLED   1

/* dh_dtype */
#define ADWIN_DT_BF16  0
#define ADWIN_DT_F32   1

/* most candidate windows one call can audit */
#define ADWIN_MAX_CANDIDATES 16

/* bits of *status_dev (device-detected input faults; the call still completes) */
#define ADWIN_DEV_BAD_ID     1u  /* some ids[t] on a computed row is outside [0, V): c_t = 0 there */
#define ADWIN_DEV_NONFINITE  2u  /* a computed row produced a non-finite log-sum-exp, mean or KL:  */
                                 /* that row is EXCLUDED -- its KL_t, c_t, diagnostics and          */
                                 /* gradient rows are written as 0 and it adds 0 to every window    */
                                 /* loss, batch value, alignment and head-weight gradient, so all   */
                                 /* outputs stay finite -- and this bit tells the caller that the   */
                                 /* Sec. 4.1 loss of the batch is short of those rows.  What to do: */
                                 /* under the single-sweep scheme (below) the cause may be a row    */
                                 /* whose logits lie more than ~80 nats above its fixed reference;  */
                                 /* call again with scheme = ADWIN_SCHEME_TWO_SWEEP, which has no   */
                                 /* such limit.  If the bit is still set, the inputs themselves     */
                                 /* hold an inf or NaN (or logits beyond the fp32 range).           */

/* scheme: how the fused path orders its passes over the vocabulary (Eq. 2 needs every row's
 * log-sum-exp and mean before Eq. 4's gradient can be formed)
 *   AUTO        SINGLE where the shape allows it (H_s >= 128 and H_t >= 128), else TWO_SWEEP_REG
 *   SINGLE      one sweep: exponentials are taken against per-row references fixed beforehand
 *               (the largest logit among the first 128 vocabulary entries and the sampled
 *               token), two gradient factors per logit are kept and combined once the row's
 *               mean is known.  Fastest; logits more than ~80 nats above the reference overflow
 *               (the row is then excluded and ADWIN_DEV_NONFINITE set).  ADWIN_E_MODE if the
 *               shape does not allow it.
 *   TWO_SWEEP   running-maximum statistics over the vocabulary, then the logits again for the
 *               gradient: any finite logit range; 1.75x the matrix work.  The diagnostics
 *               (t_*), the sampled estimator and dW_* are not offered (ADWIN_E_MODE).
 *   TWO_SWEEP_REG  TWO_SWEEP with operand tiles staged through registers, the kernel that hidden
 *               sizes of 64 need; any shape.
 * adwin_opd_workspace_bytes and adwin_opd_fused read the scheme from the same struct, so the
 * size and the call agree by construction. */
#define ADWIN_SCHEME_AUTO           0
#define ADWIN_SCHEME_SINGLE         1
#define ADWIN_SCHEME_TWO_SWEEP      2
#define ADWIN_SCHEME_TWO_SWEEP_REG  3

/* scheme of the logits-given path: which kernel streams the rows
 *   AUTO / RESIDENT  one workgroup per row keeps the row pair on chip between its two sweeps, so
 *                    memory sees each logit once (the diagnostics t_* always take STREAMING)
 *   STREAMING        reads the row pair twice; no limit on what stays resident */
#define ADWIN_LOGITS_AUTO       0
#define ADWIN_LOGITS_RESIDENT   1
#define ADWIN_LOGITS_STREAMING  2

/*
 * Problem description for the fused path (hidden states in, Sec. 4.1 / 4.2).
 * Limits: 1 <= B; 0 <= T < 2^31; V a positive multiple of 8; H_s and H_t positive
 * multiples of 64 (the k-extent of one staged MFMA tile).
 * The sampled estimator, the diagnostics (t_*) and the head-weight gradients (dW_*) ride on
 * the single-sweep kernels, which need H_s >= 128 and H_t >= 128; with a smaller hidden size, or
 * with a two-sweep `scheme`, a call that asks for them returns ADWIN_E_MODE.
 * Precision of dh_*: the logit gradient is contracted with W_s as bf16, except for the few
 * entries of a row that carry a probability of 1/32 or more, which are taken in fp32 (so that
 * peaked rows, where a handful of entries make up the gradient, are as accurate as flat ones):
 * max |dh - exact| <= 2e-3 max |dh| for vocabularies of a thousand entries or more.  Below
 * that an element sums too few terms for the roundings to average out and is off by up to
 * ~2^-8 of the Euclidean norm of its own summands instead.
 * The environment variables ADWIN_SLAB_ROWS, ADWIN_STRIPS, ADWIN_STRIPS2 and ADWIN_TG override
 * launch geometry (tuning and tests only; results do not depend on them beyond rounding order;
 * a workspace sized under one setting and used under another is refused with
 * ADWIN_E_WORKSPACE if it is too small).
 * Outputs are optional (NULL = not wanted).  When none of the requested outputs depends on
 * the gradients -- only kl, c, the window losses, n_out / n_adm_out / status_dev, the
 * diagnostics and their summaries, and batch in mode PREFIX_ONLY -- the call is a forward-only
 * statistics pass: no gradient factor is stored or contracted, and the workspace is smaller
 * accordingly (adwin_opd_workspace_bytes looks at the same pointers).
 */
typedef struct adwin_opd_problem {
  size_t  struct_bytes;      /* sizeof(adwin_opd_problem), checked                            */
  int64_t T;                 /* packed rows                                                    */
  int32_t B, V, H_s, H_t;
  const int64_t* offsets;    /* host  [B+1]  offsets[0]==0, non-decreasing, offsets[B]==T      */
  const int32_t* window;     /* host  [B]    >= 0 ; n_i = min(window[i], len_i)                */
  const void* h_s;           /* device bf16 [T, H_s]                                           */
  const void* h_t;           /* device bf16 [T, H_t]                                           */
  const void* W_s;           /* device bf16 [V, H_s]  (LM head, z = W h, no bias)              */
  const void* W_t;           /* device bf16 [V, H_t]                                           */
  const int32_t* ids;        /* device [T] sampled token y_t; may be NULL (then c is zero)     */
  int32_t mode;              /* ADWIN_PREFIX_ONLY | ADWIN_PREFIX_AND_FULL                      */
  int32_t reduction;         /* ADWIN_RED_*                                                    */
  float   grad_scale;        /* extra multiplier on dh_prefix / dh_full                        */
  int32_t dh_dtype;          /* ADWIN_DT_BF16 | ADWIN_DT_F32: element type of dh_*             */
  /* device outputs; NULL = not wanted */
  float* kl;                 /* [T] KL_t, 0 on rows not computed                               */
  float* c;                  /* [T] c_t,  0 on rows not computed or when ids==NULL             */
  void*  dh_prefix;          /* [T, H_s] grad_scale*alpha^p_i*g_t on admitted rows, else 0      */
  void*  dh_full;            /* [T, H_s] grad_scale*alpha^f_i*g_t (mode PREFIX_AND_FULL only)   */
  float* loss_prefix;        /* [B] mean KL over the window (0 if n_i == 0)                    */
  float* loss_full;          /* [B] mean KL over the rollout (zeros in PREFIX_ONLY)            */
  float* rho_pooled;         /* [B] cos(sum_t dh_prefix[t], sum_t dh_full[t]) over rollout i    */
  float* rho_field;          /* [B] cos of the two [len_i, H_s] gradient arrays of rollout i    */
  float* batch;              /* [8] L^p, L^f, pooled micro, field micro, pooled macro, field   */
                             /*     macro, head-block cosine (see dW_full), 0; the alignment    */
                             /*     entries are zero in PREFIX_ONLY                            */
  int32_t* n_out;            /* [B] n_i                                                        */
  int64_t* n_adm_out;        /* [1] N_adm = sum n_i                                            */
  uint32_t* status_dev;      /* [1] OR of ADWIN_DEV_* bits                                     */
  /* Candidate-window audit (Sec. 4.2: rho_t(L) for every L of the candidate list, all from
   * the one full-rollout pass of this call; mode PREFIX_AND_FULL only).  For candidate L
   * the prefix objective uses the shared window L on every rollout (n_i = min(L, len_i),
   * weights by `reduction`) and is compared with the same full-rollout gradient as above.
   * candidates == NULL or n_candidates == 0: no audit, the three outputs are not touched. */
  const int32_t* candidates; /* host [n_candidates], each > 0                                  */
  int32_t n_candidates;      /* 0 .. ADWIN_MAX_CANDIDATES                                      */
  float* cand_rho_pooled;    /* [n_candidates, B] per-rollout pooled cosine                     */
  float* cand_rho_field;     /* [n_candidates, B] per-rollout field cosine                      */
  float* cand_batch;         /* [n_candidates, 4] pooled micro, field micro, pooled macro,     */
                             /*                   field macro                                  */
  /* Teacher-side drift diagnostics of Sec. 3.1, per computed row (0 on the others); NULL =
   * not wanted.  The entropy and the rank add about 5 % to the vocabulary sweep. */
  float* t_logp;             /* [T] log p_t(y_t) (needs ids; 0 for an id outside [0, V))        */
  float* t_entropy;          /* [T] H[p_t] in nats; the branching factor is exp(H)              */
  int32_t* t_rank;           /* [T] 1 + number of entries the teacher ranks strictly above y_t  */
                             /*     (needs ids; 0 for an id outside [0, V))                     */
  int32_t estimator;         /* ADWIN_EST_EXPECTED | ADWIN_EST_SAMPLED                          */
  /* Gradients of the batch objectives with respect to the student LM-head weights (z = W h):
   * sum_t grad_scale * alpha_i * dz_t^T h_s[t], the third contraction of the LM-head backward.
   * NULL = not wanted; each costs one more 2 V H_s FLOP per token.  Device, 16-byte aligned
   * (else ADWIN_E_ALIGN), overwritten in full (zeros when no row is computed).  dz is the
   * logit gradient of the selected estimator.  dW_full only in mode PREFIX_AND_FULL, and
   * neither with the two-sweep fallback scheme (else ADWIN_E_MODE).  Each element
   * is a sum over rows of products whose dz factor is rounded to bf16.  With both requested,
   * batch[6] = cos(dW_prefix, dW_full): Sec. 4.2's alignment taken in the LM-head parameter
   * block (0 if either is zero). */
  float* dW_prefix;          /* [V, H_s] prefix-window objective                                */
  float* dW_full;            /* [V, H_s] full-rollout objective (mode PREFIX_AND_FULL only)     */
  /* Rollout-level summaries of the per-row outputs over each rollout's computed positions
   * (j < n_i; every position in mode PREFIX_AND_FULL).  Device pointers, NULL = not wanted.
   * t_first_reject: Sec. 3.1 top-k rejection -- the survival fraction S_T^(k) is the share of
   *   rollouts whose first rejection is at or beyond T.  Needs t_rank (else ADWIN_E_NULL) and
   *   topk > 0 (else ADWIN_E_SHAPE).
   * t_logp_mean: mean teacher log-probability of the sampled tokens inside the window and
   *   beyond it (App. C, cascading effect on the suffix); an empty region gives 0.  Needs t_logp.
   * cand_loss_share: share of the summed KL of all rows that lies on positions j < L_k, the
   *   cumulative loss distribution over positions (App. C) read at the candidate windows;
   *   0 when the total is 0.  Needs candidates (mode PREFIX_AND_FULL). */
  int32_t topk;              /* k of the top-k rejection                                       */
  int32_t* t_first_reject;   /* [B] first position j (0-based) with t_rank > topk; the number   */
                             /*     of computed positions of the rollout if there is none      */
  float* t_logp_mean;        /* [B + 1, 2] per rollout: window, beyond; row B: over all tokens  */
  float* cand_loss_share;    /* [n_candidates]                                                  */
  int32_t scheme;            /* ADWIN_SCHEME_*                                                  */
} adwin_opd_problem;

/*
 * Problem description for the logits-given path: log-softmax, reverse KL and the
 * loss gradient with respect to the student logits, no LM-head contraction.
 * Admitted rows only (Sec. 4.1).  Limits as above; V a positive multiple of 8.
 */
typedef struct adwin_opd_logits_problem {
  size_t  struct_bytes;
  int64_t T;
  int32_t B, V;
  const int64_t* offsets;    /* host [B+1]                                                     */
  const int32_t* window;     /* host [B]                                                       */
  const void* z_s;           /* device bf16 [T, V] student logits                              */
  const void* z_t;           /* device bf16 [T, V] teacher logits                              */
  const int32_t* ids;        /* device [T] or NULL                                             */
  int32_t reduction;
  float   grad_scale;
  float* kl;                 /* [T]                                                            */
  float* c;                  /* [T]                                                            */
  void*  dz;                 /* device bf16 [T, V]: grad_scale*alpha^p_i*p_s*((z_s-z_t)-mu_t)   */
                             /* on admitted rows, 0 elsewhere                                  */
  float* loss_prefix;        /* [B]                                                            */
  float* batch;              /* [8] L^p then zeros                                             */
  int32_t* n_out;            /* [B]                                                            */
  int64_t* n_adm_out;        /* [1]                                                            */
  uint32_t* status_dev;      /* [1]                                                            */
  /* teacher-side drift diagnostics of Sec. 3.1 (see adwin_opd_problem); NULL = not wanted      */
  float* t_logp;             /* [T]                                                            */
  float* t_entropy;          /* [T]                                                            */
  int32_t* t_rank;           /* [T]                                                            */
  int32_t estimator;         /* ADWIN_EST_EXPECTED | ADWIN_EST_SAMPLED: what dz carries         */
  /* rollout-level summaries over the admitted positions (see adwin_opd_problem)                */
  int32_t topk;              /* > 0 when t_first_reject is wanted                              */
  int32_t* t_first_reject;   /* [B] needs t_rank                                               */
  float* t_logp_mean;        /* [B + 1, 2] needs t_logp; the second column is 0 on this path    */
  int32_t scheme;            /* ADWIN_LOGITS_*                                                  */
} adwin_opd_logits_problem;

/* Library version: major*10000 + minor*100 + patch.  Pure host. */
int adwin_opd_version(void);

/*
 * Optional per-device set-up: sets the kernel attributes (dynamic LDS sizes) of every kernel
 * on the current HIP device and looks up the address of the static scratch array there.  The entry points do this themselves on their first call on a
 * device; a caller that captures its first call in a HIP graph, or that makes first calls
 * from several threads at once, calls this once per device beforehand.  Idempotent; no
 * memory is allocated, nothing is enqueued.  Returns ADWIN_OK or ADWIN_E_HIP.
 */
int adwin_opd_init(void);

/* Static, NUL-terminated description of a status code.  Pure host. */
const char* adwin_opd_strerror(int status);

/*
 * Integer bookkeeping of Sec. 4.1 on the host (no GPU needed): validates T, B,
 * offsets, window and writes
 *   n[B]          n_i = min(window[i], len_i)
 *   row_list[N]   packed indices of the admitted rows, ascending   (may be NULL)
 *   row_seq[N]    rollout of each admitted row                     (may be NULL)
 *   *n_adm        N = sum n_i
 * row_list / row_seq must have room for min(T, sum window) entries; call once with
 * both NULL to learn N.  All pointers are host memory.
 */
int adwin_opd_plan_host(int64_t T, int32_t B, const int64_t* offsets, const int32_t* window,
                        int32_t* n, int64_t* row_list, int32_t* row_seq, int64_t* n_adm);

/*
 * Scheduler of Sec. 4.2 (host, no GPU).
 *   snr:          Eq. 10, snr[k] = rho[k]^2 / (1 - rho[k]^2)  (+inf at |rho| = 1).
 *   next_window:  L_next = the shortest candidate whose alignment reaches rho_star; if none
 *                 does, the longest candidate (the window expands).  rho_star <= 0 selects
 *                 the paper's threshold sqrt(2)/2, the point where the SNR is 1.
 *   probe_staleness: bookkeeping of the hard staleness limit of Sec. 4.1.  Called once
 *                 per optimisation step: the age of every pending probe (pending[i] != 0)
 *                 grows by one, ages of the others are reset to 0; force[i] = 1 for the
 *                 pending probes whose age has reached `limit` (paper: 5), which must be
 *                 completed before the next step.  *n_forced counts them.
 * All pointers are host memory; rho, candidates: [k]; age, pending, force: [n_probes].
 */
int adwin_opd_snr(const float* rho, int32_t k, float* snr);
int adwin_opd_next_window(const float* rho, const int32_t* candidates, int32_t k, float rho_star,
                          int32_t* next);
int adwin_opd_probe_staleness(int32_t* age, const uint8_t* pending, int32_t n_probes, int32_t limit,
                              uint8_t* force, int32_t* n_forced);

/* Bytes of device workspace adwin_opd_fused needs for this problem.  Pure host; reads
 * shapes, mode, offsets and window only. */
int adwin_opd_workspace_bytes(const adwin_opd_problem* p, size_t* bytes);

/* Launch geometry adwin_opd_fused will use for this problem (pure host; for benchmarks that
 * quote per-launch figures): info[0] = rows computed, info[1] = the same padded to whole
 * 256-row tiles, info[2] = rows per slab (the sweep and the gradient GEMM are launched once
 * per slab), info[3] = number of slabs. */
int adwin_opd_fused_launch_info(const adwin_opd_problem* p, int64_t info[4]);

/*
 * Fused path (Sec. 4.1 loss on the prefix; Sec. 4.2 probe audit in mode
 * PREFIX_AND_FULL): LM-head projections, full-vocabulary log-softmax, KL_t, c_t,
 * g_t, window losses, dh_prefix / dh_full and the alignment scores.  The [rows, V]
 * logit matrix is never stored.  `workspace` is device memory, 256-byte aligned,
 * at least adwin_opd_workspace_bytes() long; its contents are scratch.
 */
int adwin_opd_fused(const adwin_opd_problem* p, void* workspace, size_t workspace_bytes,
                    void* hip_stream);

/* Bytes of device workspace adwin_opd_from_logits needs.  Pure host. */
int adwin_opd_logits_workspace_bytes(const adwin_opd_logits_problem* p, size_t* bytes);

/*
 * Logits-given path: same per-token mathematics with z_s, z_t read from memory
 * (Eq. 2 at token level, c_t, and the logit gradient of Eq. 4 in expectation),
 * followed by the window losses.  Bandwidth-bound.
 */
int adwin_opd_from_logits(const adwin_opd_logits_problem* p, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

/*
 * adwin_opd_from_logits for callers that cannot allocate device memory or size a workspace:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, checks, kernels and results as adwin_opd_from_logits, but the scratch (plan
 * arrays, a KL copy per row, per-rollout accumulators) lives in a fixed array of
 * ADWIN_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held until the process ends;
 * the call itself allocates nothing, on the device or through any library.  A problem whose
 * adwin_opd_logits_workspace_bytes() exceeds that size is refused with ADWIN_E_WORKSPACE and
 * nothing is enqueued (1 MiB covers T + 60 B up to about 260,000: e.g. 32 rollouts of 8,192
 * rows).  Inputs and outputs are the caller's, as always.  Every call on a GPU uses that GPU's
 * one array: calls that overlap in time on the same GPU (different streams, or threads) race
 * and give undefined results; calls on one stream, or ordered by events, are fine, and nothing
 * one call leaves in the array is read by the next.  The array's address is looked up on the
 * first call on a device, or by adwin_opd_init: a caller that captures its first call in a HIP
 * graph calls adwin_opd_init beforehand.
 */
#define ADWIN_STATIC_SCRATCH_BYTES (1 << 20)
int adwin_opd_from_logits_static(const adwin_opd_logits_problem* p, void* hip_stream);

/*
 * Profiling variants: identical work and results, but every kernel launch is bracketed
 * with HIP events on the stream, the call waits for the stream to drain, and the summed
 * milliseconds per phase are written to phase_ms (host float[ADWIN_N_PHASES]).  Phases
 * follow the steps of the path: setup (plan upload, W_s transpose), full-vocabulary
 * statistics pass (Eq. 2 terms), per-row merge (KL_t, c_t), logit-gradient pass (Eq. 4 in
 * expectation), gradient contraction with W_s, and scatter plus window reductions
 * (Sec. 4.1 losses, Sec. 4.2 alignment).  The logits-given variant reports its single
 * streaming kernel under ADWIN_PHASE_STATS and the reductions under ADWIN_PHASE_REDUCE.
 */
#define ADWIN_PHASE_SETUP   0
#define ADWIN_PHASE_STATS   1
#define ADWIN_PHASE_MERGE   2
#define ADWIN_PHASE_DZ      3
#define ADWIN_PHASE_GRAD    4
#define ADWIN_PHASE_REDUCE  5
#define ADWIN_N_PHASES      6
int adwin_opd_fused_profile(const adwin_opd_problem* p, void* workspace, size_t workspace_bytes,
                            void* hip_stream, float* phase_ms);
int adwin_opd_from_logits_profile(const adwin_opd_logits_problem* p, void* workspace,
                                  size_t workspace_bytes, void* hip_stream, float* phase_ms);

/*
 * Measured ceilings of the machine, for quoting roofline fractions against what the box
 * delivers as well as against the published peaks.  Both synchronise.
 *   copy: streams `bytes` (multiple of 16; device pointers, 16-byte aligned) from src to
 *         dst `reps` times; *ms (host) = average milliseconds per copy.
 *   mfma: register-resident v_mfma_f32_32x32x16_bf16 loop on every CU; `scratch` is at
 *         least 4 bytes of device memory; *tflops (host) = achieved dense bf16 TFLOP/s.
 */
int adwin_opd_ceiling_copy(const void* src, void* dst, size_t bytes, int reps, void* hip_stream,
                           float* ms);
int adwin_opd_ceiling_mfma(void* scratch, int iters, void* hip_stream, float* tflops);
/* The same loop with pseudo-random operands (signs, mantissas and exponents vary from
 * lane to lane as in real inputs): the matrix-core rate the power limit sustains on such
 * data, below the constant-operand figure.  Synchronises. */
int adwin_opd_ceiling_mfma_random(void* scratch, int iters, void* hip_stream, float* tflops);

#ifdef __cplusplus
}
#endif
#endif /* ADWIN_OPD_H */
