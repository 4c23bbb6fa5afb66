"""Rounding-error model of a reduced-precision logit gradient: test machinery, not part of
the oracle and not the paper's definition.

An implementation that stores the logit gradient dz_t of Eq. 4 (in expectation: p_s (Delta -
KL_t)) as bf16, built from separately rounded factors p_s and a centred Delta, makes errors
proportional to p_s (|Delta - KL_t| + D_t) per entry, D_t the standard deviation of Delta under
p_s, and not to |dz_t|, which vanishes wherever Delta happens to equal KL_t.  A gradient element
that sums such entries (g = dz W_s over the vocabulary, dW = sum over rows of w dz^T h_s) then
errs by about 2^-9 times the Euclidean norm of its summands taken at that scale.  The tests use
these norms for per-element bounds where a fraction of the largest element says nothing:
vocabularies of a few hundred entries, and the head-weight gradient.

Everything here is computed with scipy's log-softmax from the same fp64 inputs the oracle
takes; nothing is imported from the oracle or from the GPU package."""
import numpy as np
import scipy.special

EST_EXPECTED, EST_SAMPLED = 0, 1


def dz_scale(z_s, z_t):
    """p_s (|Delta - KL_t| + D_t) per vocabulary entry."""
    ls, lt = scipy.special.log_softmax(z_s), scipy.special.log_softmax(z_t)
    p = np.exp(ls)
    delta = ls - lt
    kl = np.sum(p * delta)
    dev = np.sqrt(np.sum(p * (delta - kl) ** 2))
    return p * (np.abs(delta - kl) + dev)


def dz_sampled_scale(z_s, z_t, y):
    """|c_t| p_s off the sampled entry and |c_t| on it: the entry c_t (1 - p_s(y_t)) is a
    difference of two rounded terms of magnitude up to |c_t| and vanishes as p_s(y_t) -> 1
    while their errors do not."""
    ls, lt = scipy.special.log_softmax(z_s), scipy.special.log_softmax(z_t)
    c = abs(ls[y] - lt[y])
    s = c * np.exp(ls)
    s[y] = c
    return s


def _scales(H_s, H_t, W_s, W_t, ids, estimator):
    Z_s, Z_t = H_s @ W_s.T, H_t @ W_t.T
    if estimator == EST_EXPECTED:
        return np.stack([dz_scale(Z_s[r], Z_t[r]) for r in range(len(Z_s))])
    return np.stack([dz_sampled_scale(Z_s[r], Z_t[r], int(ids[r])) for r in range(len(Z_s))])


def hidden_summand_norms(H_s, H_t, W_s, W_t, ids=None, estimator=EST_EXPECTED, block=64):
    """[K, H_s]: sqrt(sum_v (s_r[v] W_s[v][k])^2) for every row r of the stack."""
    out = np.zeros((H_s.shape[0], W_s.shape[1]))
    W2 = W_s ** 2
    for r0 in range(0, H_s.shape[0], block):
        r1 = min(H_s.shape[0], r0 + block)
        S = _scales(H_s[r0:r1], H_t[r0:r1], W_s, W_t, None if ids is None else ids[r0:r1], estimator)
        out[r0:r1] = np.sqrt((S ** 2) @ W2)
    return out


def head_summand_norms(H_s, H_t, W_s, W_t, weights, ids=None, estimator=EST_EXPECTED, block=64):
    """For each per-row weight vector w of `weights`, [V, H_s]:
    sqrt(sum_r (w[r] s_r[v] h_s[r][k])^2)."""
    acc = [np.zeros(W_s.shape) for _ in weights]
    for r0 in range(0, H_s.shape[0], block):
        r1 = min(H_s.shape[0], r0 + block)
        S = _scales(H_s[r0:r1], H_t[r0:r1], W_s, W_t, None if ids is None else ids[r0:r1], estimator)
        for k, w in enumerate(weights):
            wS = S * np.asarray(w)[r0:r1, None]
            acc[k] += (wS ** 2).T @ (H_s[r0:r1] ** 2)
    return [np.sqrt(a) for a in acc]


def problem_norms(f, offsets, window, rows, alpha_p, alpha_f, grad_scale=1.0, estimator=EST_EXPECTED,
                  head=False, block=64):
    """Summand norms for a whole problem.  f: dict of fp64 inputs (h_s, h_t, W_s, W_t, ids);
    rows: the packed rows the mode computes; alpha_p / alpha_f: per-rollout weights of the
    reduction.  Returns g_l2 [T, H_s] (0 on rows not computed) and, with head, dW_prefix_l2 and
    dW_full_l2."""
    T = int(offsets[-1])
    B = len(window)
    lens = np.diff(offsets)
    n = np.minimum(np.asarray(window, np.int64), lens)
    ids = f.get("ids")
    rows = np.asarray(rows, np.int64)
    g_l2 = np.zeros((T, f["W_s"].shape[1]))
    out = {"g_l2": g_l2}
    if len(rows) == 0:
        if head:
            out["dW_prefix_l2"] = np.zeros(f["W_s"].shape)
            out["dW_full_l2"] = np.zeros(f["W_s"].shape)
        return out
    rid = None if ids is None else np.asarray(ids)[rows]
    g_l2[rows] = hidden_summand_norms(f["h_s"][rows], f["h_t"][rows], f["W_s"], f["W_t"], rid, estimator, block)
    if head:
        wp, wf = np.zeros(T), np.zeros(T)
        for i in range(B):
            o = int(offsets[i])
            wp[o:o + int(n[i])] = grad_scale * alpha_p[i]
            wf[o:o + int(lens[i])] = grad_scale * alpha_f[i]
        l2 = head_summand_norms(f["h_s"][rows], f["h_t"][rows], f["W_s"], f["W_t"], [wp[rows], wf[rows]],
                                rid, estimator, block)
        out["dW_prefix_l2"], out["dW_full_l2"] = l2
    return out
