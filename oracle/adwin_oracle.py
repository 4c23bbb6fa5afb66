"""fp64 CPU oracle for teacher-anchored per-token supervision over ragged rollouts.

TEST INFRASTRUCTURE ONLY.  This file defines, as slowly and plainly as possible,
what the GPU library must compute.  Only the tests, the smoke check and the
benchmark's `cpu_baseline` leg may import it; it shares no code with the HIP path
and imports nothing from the product package.

What is computed (all from the paper; where it is silent the reading is stated):

* Rollout i occupies packed rows offsets[i] .. offsets[i+1)-1.  A shared (here:
  per-rollout) window truncates supervision to the first n_i = min(window_i, len_i)
  response positions (Sec. 4.1, synchronous path: the loss is evaluated on the
  prefix only).
* Row t holds the hidden state of context (x, y_<t); logits are z = W h with no
  bias and temperature 1 (OPD hyper-parameter table: sampling temperature 1.0,
  top-p 1.0, so no rescaling or filtering of the distribution).
* Per-token loss is the token-level instance of the OPD objective (Eq. 2):
  KL(pi_theta(.|s_t) || pi_phi(.|s_t)), student first, teacher frozen.
* The sampled step cost is c_t = log pi_theta(y_t|s_t) - log pi_phi(y_t|s_t)
  (Sec. 2.3 and App. A.1).
* The gradient is the one of the gamma = 0 token-local estimator (Eq. 4) in
  expectation over y_t ~ pi_theta: E[c_t (e_y - p_s)] = p_s (Delta - KL_t), which is
  also d KL_t / d z_s with the teacher held fixed (App. A.1: teacher is constant,
  expected score is zero).  Back to the hidden state: g_t = dz_t W_s.
* Alignment is the cosine between the prefix-window gradient and the full-rollout
  gradient (Sec. 4.2), per rollout and after batch aggregation ("macro" / "micro",
  Fig. 5 caption).

Readings where the paper is silent: loss inside a window is the token mean and the
batch loss is the mean over rollouts (`RED_SEQ_MEAN`); sum and token-mean are
selectable.  The gradient space of the cosine is dL/dh_s: "pooled" sums a rollout's
per-token gradients into one H_s-vector (what a parameter shared across positions
would receive), "field" is the literal cosine of the two [len_i, H_s] gradient
arrays.  A cosine with a zero norm is 0 and is left out of the macro mean.

Every function here is pinned by tests/test_oracle_*.py against closed forms,
library routines (scipy), finite differences and brute-force enumeration.
"""
from __future__ import annotations

import numpy as np

RED_SEQ_MEAN = 0
RED_SUM = 1
RED_TOKEN_MEAN = 2

MODE_PREFIX_ONLY = 0
MODE_PREFIX_AND_FULL = 1

EST_EXPECTED = 0     # gradient of the full-vocabulary KL_t = expectation of Eq. 4 over y_t ~ p_s
EST_SAMPLED = 1      # Eq. 4 itself, on the sampled token y_t

RHO_STAR = np.sqrt(2.0) / 2.0          # Eq. 10
CANDIDATE_WINDOWS = (64, 128, 256, 512, 1024, 2048)   # training details, Sec. 5.1


# ---------------------------------------------------------------------------
# integer bookkeeping  (Sec. 4.1: rollouts truncated at the window)
# ---------------------------------------------------------------------------

def plan(offsets, window):
    """len_i, n_i = min(window_i, len_i), admitted packed rows (ascending), the
    rollout each admitted row belongs to, and N_adm.  Plain integer loops."""
    offsets = [int(o) for o in offsets]
    window = [int(w) for w in window]
    B = len(window)
    if len(offsets) != B + 1 or offsets[0] != 0:
        raise ValueError("offsets must have B+1 entries starting at 0")
    lens, n, rows, seq = [], [], [], []
    for i in range(B):
        l = offsets[i + 1] - offsets[i]
        if l < 0:
            raise ValueError("offsets must be non-decreasing")
        if window[i] < 0:
            raise ValueError("window must be >= 0")
        ni = window[i] if window[i] < l else l
        lens.append(l)
        n.append(ni)
        for j in range(ni):
            rows.append(offsets[i] + j)
            seq.append(i)
    return {
        "len": np.asarray(lens, np.int64),
        "n": np.asarray(n, np.int32),
        "rows": np.asarray(rows, np.int64),
        "row_seq": np.asarray(seq, np.int32),
        "n_adm": int(sum(n)),
    }


# ---------------------------------------------------------------------------
# one token  (Eq. 2 at token level, c_t of Sec. 2.3, gradient of Eq. 4 / App. A.1)
# ---------------------------------------------------------------------------

def log_softmax(z):
    z = np.asarray(z, np.float64)
    m = np.max(z)
    return z - (m + np.log(np.sum(np.exp(z - m))))


def token_kl(z_s, z_t):
    """KL(softmax(z_s) || softmax(z_t)): student first (Eq. 2)."""
    ls, lt = log_softmax(z_s), log_softmax(z_t)
    return float(np.sum(np.exp(ls) * (ls - lt)))


def token_cost(z_s, z_t, y):
    """c_t = log p_s(y) - log p_t(y)."""
    return float(log_softmax(z_s)[y] - log_softmax(z_t)[y])


def token_dz(z_s, z_t):
    """d KL_t / d z_s with the teacher fixed: p_s (Delta - KL_t)."""
    ls, lt = log_softmax(z_s), log_softmax(z_t)
    p = np.exp(ls)
    delta = ls - lt
    return p * (delta - np.sum(p * delta))


def token_dz_sampled(z_s, z_t, y):
    """The per-token term of the gamma = 0 estimator (Eq. 4) in logit space:
    c_t * d log p_s(y_t) / d z_s = c_t (e_{y_t} - p_s), with c_t held constant."""
    p = np.exp(log_softmax(z_s))
    e_y = np.zeros_like(p)
    e_y[y] = 1.0
    return token_cost(z_s, z_t, y) * (e_y - p)


def token_terms(h_s, h_t, W_s, W_t, y=None, estimator=EST_EXPECTED):
    """Logits from hidden states, then KL_t, c_t and g_t = dz_t W_s for one row."""
    z_s = W_s @ h_s
    z_t = W_t @ h_t
    kl = token_kl(z_s, z_t)
    c = token_cost(z_s, z_t, y) if y is not None else 0.0
    dz = token_dz(z_s, z_t) if estimator == EST_EXPECTED else token_dz_sampled(z_s, z_t, y)
    g = dz @ W_s
    return kl, c, g


def rows_terms(H_s, H_t, W_s, W_t, ids=None, block=16, estimator=EST_EXPECTED, head_weights=None):
    """`token_terms` for a stack of independent rows.  Rows are batched through one
    matrix product per block only to let BLAS do the inner products; each row's
    softmax/KL/gradient is the single-row definition above.

    head_weights: optional list of per-row weight vectors w; for each one the gradient of
    sum_r w[r] KL_r with respect to the student LM-head weights, sum_r w[r] dz_r^T h_s[r]
    (z = W h, so d z[v] / d W[v, k] = h[k]), is returned as a fourth value."""
    K = H_s.shape[0]
    kl = np.zeros(K)
    c = np.zeros(K)
    g = np.zeros((K, W_s.shape[1]))
    dW = None if head_weights is None else [np.zeros(W_s.shape) for _ in head_weights]
    for r0 in range(0, K, block):
        r1 = min(K, r0 + block)
        Z_s = H_s[r0:r1] @ W_s.T
        Z_t = H_t[r0:r1] @ W_t.T
        D = np.empty_like(Z_s)
        for r in range(r0, r1):
            z_s, z_t = Z_s[r - r0], Z_t[r - r0]
            kl[r] = token_kl(z_s, z_t)
            if ids is not None:
                c[r] = token_cost(z_s, z_t, int(ids[r]))
            if estimator == EST_EXPECTED:
                D[r - r0] = token_dz(z_s, z_t)
            else:
                D[r - r0] = token_dz_sampled(z_s, z_t, int(ids[r]))
        g[r0:r1] = D @ W_s
        if dW is not None:
            for k, w in enumerate(head_weights):
                wD = D * np.asarray(w)[r0:r1, None]
                dW[k] += wD.T @ H_s[r0:r1]
    if dW is not None:
        return kl, c, g, dW
    return kl, c, g


# ---------------------------------------------------------------------------
# windows, weights, alignment
# ---------------------------------------------------------------------------

def row_weights(lens, n, reduction):
    """Per-rollout weights alpha^p_i, alpha^f_i of a token's KL in the batch
    objective (prefix and full-rollout)."""
    B = len(n)
    ap, af = np.zeros(B), np.zeros(B)
    n_adm, T = int(np.sum(n)), int(np.sum(lens))
    for i in range(B):
        if reduction == RED_SEQ_MEAN:
            ap[i] = 1.0 / (B * n[i]) if n[i] > 0 else 0.0
            af[i] = 1.0 / (B * lens[i]) if lens[i] > 0 else 0.0
        elif reduction == RED_SUM:
            ap[i] = af[i] = 1.0
        elif reduction == RED_TOKEN_MEAN:
            ap[i] = 1.0 / n_adm if n_adm > 0 else 0.0
            af[i] = 1.0 / T if T > 0 else 0.0
        else:
            raise ValueError("reduction")
    return ap, af


def cosine(a, b):
    na, nb = np.sqrt(np.sum(a * a)), np.sqrt(np.sum(b * b))
    if na == 0.0 or nb == 0.0:
        return 0.0
    return float(np.sum(a * b) / (na * nb))


def window_outputs(kl, g, offsets, window, reduction=RED_SEQ_MEAN, grad_scale=1.0,
                   mode=MODE_PREFIX_AND_FULL):
    """Everything downstream of the per-token terms.

    kl[T] and g[T,H] must hold the per-token values on every row the mode computes
    (all rows in probe mode, admitted rows otherwise; other rows are ignored).
    Returns per-window losses, dh_prefix / dh_full, per-rollout and batch alignment.
    """
    p = plan(offsets, window)
    lens, n = p["len"], p["n"]
    B, T = len(n), int(offsets[-1])
    H = g.shape[1]
    ap, af = row_weights(lens, n, reduction)
    probe = mode == MODE_PREFIX_AND_FULL

    loss_p, loss_f = np.zeros(B), np.zeros(B)
    dh_p, dh_f = np.zeros((T, H)), np.zeros((T, H))
    rho_pool, rho_field = np.zeros(B), np.zeros(B)
    up_sum, uf_sum = np.zeros(H), np.zeros(H)
    macro_pool, macro_field = [], []
    Lp = Lf = 0.0
    for i in range(B):
        o = int(offsets[i])
        for j in range(int(n[i])):
            loss_p[i] += kl[o + j] / n[i]
            Lp += ap[i] * kl[o + j]
            dh_p[o + j] = grad_scale * ap[i] * g[o + j]
        if probe:
            for j in range(int(lens[i])):
                loss_f[i] += kl[o + j] / lens[i]
                Lf += af[i] * kl[o + j]
                dh_f[o + j] = grad_scale * af[i] * g[o + j]
            sl = slice(o, o + int(lens[i]))
            u_p = dh_p[sl].sum(axis=0)           # pooled prefix gradient
            u_f = dh_f[sl].sum(axis=0)           # pooled full-rollout gradient
            rho_pool[i] = cosine(u_p, u_f)
            rho_field[i] = cosine(dh_p[sl].ravel(), dh_f[sl].ravel())
            if np.any(u_p != 0.0) and np.any(u_f != 0.0):
                macro_pool.append(rho_pool[i])
            if np.any(dh_p[sl] != 0.0) and np.any(dh_f[sl] != 0.0):
                macro_field.append(rho_field[i])
            up_sum += u_p
            uf_sum += u_f
    batch = np.zeros(8)
    batch[0] = Lp
    if probe:
        batch[1] = Lf
        batch[2] = cosine(up_sum, uf_sum)                  # micro: after batch aggregation
        batch[3] = cosine(dh_p.ravel(), dh_f.ravel())
        batch[4] = float(np.mean(macro_pool)) if macro_pool else 0.0   # macro: mean of
        batch[5] = float(np.mean(macro_field)) if macro_field else 0.0  # per-rollout cosines
    return {
        "n": n, "n_adm": p["n_adm"],
        "loss_prefix": loss_p, "loss_full": loss_f,
        "dh_prefix": dh_p, "dh_full": dh_f,
        "rho_pooled": rho_pool, "rho_field": rho_field, "batch": batch,
    }


def supervise(h_s, h_t, W_s, W_t, ids, offsets, window, reduction=RED_SEQ_MEAN,
              grad_scale=1.0, mode=MODE_PREFIX_ONLY, estimator=EST_EXPECTED, head_gradient=False,
              block=16):
    """Whole path from hidden states (fp64 arrays holding the bf16-exact inputs).
    head_gradient: also dW_prefix / dW_full, the gradients of the prefix and full-rollout
    batch objectives (times grad_scale) with respect to the student LM-head weights.
    block: rows per library matrix product in `rows_terms` (batching only)."""
    p = plan(offsets, window)
    T = int(offsets[-1])
    if mode == MODE_PREFIX_AND_FULL:
        rows = np.arange(T, dtype=np.int64)
    else:
        rows = p["rows"]
    kl, c, g = np.zeros(T), np.zeros(T), np.zeros((T, W_s.shape[1]))
    dW = None
    hw = None
    if head_gradient:
        ap, af = row_weights(p["len"], p["n"], reduction)
        wp, wf = np.zeros(T), np.zeros(T)
        for i in range(len(p["n"])):
            o = int(offsets[i])
            wp[o:o + int(p["n"][i])] = grad_scale * ap[i]
            wf[o:o + int(p["len"][i])] = grad_scale * af[i]
        hw = [wp[rows], wf[rows]]
    if len(rows):
        res = rows_terms(h_s[rows], h_t[rows], W_s, W_t,
                         None if ids is None else np.asarray(ids)[rows], block=block,
                         estimator=estimator, head_weights=hw)
        kl[rows], c[rows], g[rows] = res[0], res[1], res[2]
        if head_gradient:
            dW = res[3]
    out = window_outputs(kl, g, offsets, window, reduction, grad_scale, mode)
    out.update(kl=kl, c=c, g=g, rows=rows)
    if head_gradient:
        zero = np.zeros(W_s.shape)
        out["dW_prefix"] = dW[0] if dW is not None else zero
        out["dW_full"] = (dW[1] if dW is not None else zero) if mode == MODE_PREFIX_AND_FULL else zero
        # alignment of the two objectives in the LM-head parameter block (Sec. 4.2's cosine taken
        # over the one parameter block this path differentiates)
        out["rho_head"] = cosine(out["dW_prefix"].ravel(), out["dW_full"].ravel())
    return out


def supervise_from_logits(z_s, z_t, ids, offsets, window, reduction=RED_SEQ_MEAN,
                          grad_scale=1.0, estimator=EST_EXPECTED):
    """Logits-given variant: per-token KL and c on admitted rows, the loss gradient
    with respect to the student logits dz[t] = grad_scale * alpha^p_i * p_s (Delta-KL),
    and the prefix-window losses.  Rows outside the windows are zero."""
    p = plan(offsets, window)
    lens, n = p["len"], p["n"]
    T, V = z_s.shape
    ap, _ = row_weights(lens, n, reduction)
    kl, c, dz = np.zeros(T), np.zeros(T), np.zeros((T, V))
    loss_p = np.zeros(len(n))
    Lp = 0.0
    for t, i in zip(p["rows"], p["row_seq"]):
        kl[t] = token_kl(z_s[t], z_t[t])
        if ids is not None:
            c[t] = token_cost(z_s[t], z_t[t], int(ids[t]))
        if estimator == EST_EXPECTED:
            dz[t] = grad_scale * ap[i] * token_dz(z_s[t], z_t[t])
        else:
            dz[t] = grad_scale * ap[i] * token_dz_sampled(z_s[t], z_t[t], int(ids[t]))
        loss_p[i] += kl[t] / n[i]
        Lp += ap[i] * kl[t]
    batch = np.zeros(8)
    batch[0] = Lp
    return {"n": n, "n_adm": p["n_adm"], "kl": kl, "c": c, "dz": dz,
            "loss_prefix": loss_p, "batch": batch}


# ---------------------------------------------------------------------------
# audit over candidate windows and the scheduler  (Sec. 4.2)
# ---------------------------------------------------------------------------

def audit_candidates(g, offsets, candidates=CANDIDATE_WINDOWS, reduction=RED_SEQ_MEAN):
    """rho_t(L) for every candidate L from one full-rollout pass: per-rollout pooled and
    field cosines [len(candidates), B], their macro means, and the micro
    (batch-aggregated) cosines, each prefix gradient (shared window L on every rollout)
    compared with the full-rollout gradient."""
    B = len(offsets) - 1
    K = len(candidates)
    per, per_field = np.zeros((K, B)), np.zeros((K, B))
    micro, macro = np.zeros(K), np.zeros(K)
    micro_field, macro_field = np.zeros(K), np.zeros(K)
    for k, L in enumerate(candidates):
        w = np.full(B, L, np.int64)
        out = window_outputs(np.zeros(int(offsets[-1])), g, offsets, w, reduction,
                             1.0, MODE_PREFIX_AND_FULL)
        per[k] = out["rho_pooled"]
        per_field[k] = out["rho_field"]
        micro[k] = out["batch"][2]
        micro_field[k] = out["batch"][3]
        macro[k] = out["batch"][4]
        macro_field[k] = out["batch"][5]
    return {"rho_pooled": per, "rho_field": per_field, "micro": micro, "macro": macro,
            "micro_field": micro_field, "macro_field": macro_field}


def snr(rho):
    """SNR_t(L) = rho^2 / (1 - rho^2)."""
    return rho * rho / (1.0 - rho * rho)


def next_window(rho_by_candidate, candidates=CANDIDATE_WINDOWS, rho_star=RHO_STAR):
    """L_{t+1} = shortest candidate whose alignment reaches rho*.  If none does the
    window expands to the longest candidate (the paper only says it expands)."""
    order = np.argsort(np.asarray(candidates))
    for k in order:
        if rho_by_candidate[k] >= rho_star:
            return int(candidates[k])
    return int(max(candidates))


# ---------------------------------------------------------------------------
# teacher-side drift diagnostics  (Sec. 3.1)
# ---------------------------------------------------------------------------

def teacher_branching_factor(z_t):
    """BF_t = exp(H[pi_phi(.|y_<t)])."""
    lt = log_softmax(z_t)
    return float(np.exp(-np.sum(np.exp(lt) * lt)))


def teacher_entropy(z_t):
    """H[pi_phi(.|y_<t)] in nats (the logarithm of the branching factor)."""
    lt = log_softmax(z_t)
    return float(-np.sum(np.exp(lt) * lt))


def teacher_logp(z_t, y):
    """log pi_phi(y_t | y_<t): the teacher's log-probability of the sampled token."""
    return float(log_softmax(z_t)[y])


def teacher_rank(z_t, y):
    """Rank of y under the teacher distribution, 1 = most likely (ties: strictly
    greater logits count)."""
    return int(np.sum(np.asarray(z_t) > z_t[y])) + 1


def topk_survival(ranks_by_rollout, k, T):
    """S_T^(k): fraction of rollouts with every rank up to position T within top-k."""
    alive = [all(r <= k for r in ranks[:T]) for ranks in ranks_by_rollout]
    return float(np.mean(alive)) if alive else 0.0


def first_rejection(ranks, k):
    """Position (0-based) of a rollout's first top-k rejection, r_t > k; the number of positions
    if there is none.  A rollout survives through position T (Sec. 3.1) iff this is >= T."""
    for j, r in enumerate(ranks):
        if r > k:
            return j
    return len(ranks)


def region_means(values, offsets, n, computed):
    """Mean of a per-token quantity over the window (positions j < n_i) and over the rest of
    the computed positions (n_i <= j < computed_i) of every rollout -- the prefix / suffix
    split of the teacher log-probability (App. C, cascading effect) -- and, last row, the same
    over all rollouts' tokens.  An empty region has mean 0.  Returns [B + 1, 2]."""
    B = len(n)
    out = np.zeros((B + 1, 2))
    tot = np.zeros(2)
    cnt = np.zeros(2)
    for i in range(B):
        o = int(offsets[i])
        regions = ((0, int(n[i])), (int(n[i]), int(computed[i])))
        for c, (lo, hi) in enumerate(regions):
            if hi > lo:
                seg = np.asarray(values[o + lo:o + hi], dtype=np.float64)
                out[i, c] = seg.sum() / (hi - lo)
                tot[c] += seg.sum()
                cnt[c] += hi - lo
    for c in range(2):
        out[B, c] = tot[c] / cnt[c] if cnt[c] > 0 else 0.0
    return out


def loss_share(kl, offsets, computed, candidates):
    """Share of the batch's summed token loss that falls on positions j < L, for every L of
    the list: the cumulative loss distribution over response positions (App. C, loss
    distribution on prefix) read at the candidate windows.  0 when the total is 0."""
    total = 0.0
    part = np.zeros(len(candidates))
    for i in range(len(computed)):
        o, m = int(offsets[i]), int(computed[i])
        seg = np.asarray(kl[o:o + m], dtype=np.float64)
        total += seg.sum()
        for k, L in enumerate(candidates):
            part[k] += seg[:min(int(L), m)].sum()
    return part / total if total != 0.0 else np.zeros(len(candidates))
