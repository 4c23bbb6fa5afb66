"""Pins for the fp64 oracle: closed forms, library routines, finite differences,
brute-force enumeration and invariants.  None of these re-types the oracle's own
formula; each would fail under a plausible mistake (a swapped KL direction, a
dropped term, a transposed operand, an off-by-one in the window)."""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import adwin_oracle as O

RNG = np.random.default_rng(7)


# ---------------------------------------------------------------- bookkeeping

def _plan_vectorised(offsets, window):
    offsets = np.asarray(offsets, np.int64)
    lens = np.diff(offsets)
    n = np.minimum(np.asarray(window, np.int64), lens)
    seq = np.repeat(np.arange(len(n)), n)
    start = np.repeat(offsets[:-1], n)
    first = np.repeat(np.cumsum(n) - n, n)
    rows = start + (np.arange(n.sum()) - first)
    return lens, n, rows, seq


@pytest.mark.parametrize("seed", range(20))
def test_plan_matches_vectorised(seed):
    g = np.random.default_rng(seed)
    B = int(g.integers(1, 9))
    lens = g.integers(0, 40, size=B)
    lens[g.integers(0, B)] = 0 if seed % 3 == 0 else lens[0]
    window = g.integers(0, 50, size=B)
    offsets = np.concatenate([[0], np.cumsum(lens)])
    p = O.plan(offsets, window)
    l2, n2, rows2, seq2 = _plan_vectorised(offsets, window)
    assert np.array_equal(p["len"], l2)
    assert np.array_equal(p["n"], n2)
    assert np.array_equal(p["rows"], rows2)
    assert np.array_equal(p["row_seq"], seq2)
    assert p["n_adm"] == int(n2.sum()) == len(p["rows"])
    assert np.all(np.diff(p["rows"]) > 0)


def test_plan_tiny_config_values():
    p = O.plan([0, 96, 224], [64, 128])
    assert p["n"].tolist() == [64, 128] and p["n_adm"] == 192
    assert p["rows"][:64].tolist() == list(range(64))
    assert p["rows"][64:].tolist() == list(range(96, 224))     # second rollout fully covered


def test_plan_edge_cases_and_errors():
    p = O.plan([0, 0, 5, 5], [3, 0, 9])
    assert p["n"].tolist() == [0, 0, 0] and p["n_adm"] == 0 and len(p["rows"]) == 0
    p = O.plan([0, 4], [9])
    assert p["n"].tolist() == [4]
    with pytest.raises(ValueError):
        O.plan([1, 4], [2])
    with pytest.raises(ValueError):
        O.plan([0, 4, 3], [2, 2])
    with pytest.raises(ValueError):
        O.plan([0, 4], [-1])


# ---------------------------------------------------------------- softmax / KL

@pytest.mark.parametrize("V", [2, 5, 16, 257])
def test_log_softmax_and_kl_match_scipy(V):
    z_s, z_t = RNG.normal(0, 3, V), RNG.normal(0, 3, V)
    assert np.allclose(O.log_softmax(z_s), scipy.special.log_softmax(z_s), rtol=0, atol=1e-13)
    assert abs(np.exp(O.log_softmax(z_s)).sum() - 1) < 1e-13
    p, q = scipy.special.softmax(z_s), scipy.special.softmax(z_t)
    assert O.token_kl(z_s, z_t) == pytest.approx(scipy.stats.entropy(p, q), rel=1e-12)


def test_kl_direction_two_token_closed_form():
    # Bernoulli(p) vs Bernoulli(q): student first.
    a, b = 1.3, -0.4
    p, q = 1 / (1 + math.exp(-a)), 1 / (1 + math.exp(-b))
    want = p * math.log(p / q) + (1 - p) * math.log((1 - p) / (1 - q))
    other = q * math.log(q / p) + (1 - q) * math.log((1 - q) / (1 - p))
    got = O.token_kl([a, 0.0], [b, 0.0])
    assert got == pytest.approx(want, rel=1e-13)
    assert abs(got - other) > 1e-2          # the reverse direction is a different number


def test_kl_zero_nonneg_shift_invariant_large_logits():
    for _ in range(50):
        V = int(RNG.integers(2, 40))
        z_s, z_t = RNG.normal(0, 4, V), RNG.normal(0, 4, V)
        assert O.token_kl(z_s, z_s) == 0.0
        k = O.token_kl(z_s, z_t)
        assert k >= 0
        assert O.token_kl(z_s + 3.7, z_t - 11.0) == pytest.approx(k, rel=1e-12, abs=1e-14)
    # no overflow with huge logits, and the one-hot limit KL -> -log p_t(argmax)
    z_s = np.zeros(9); z_s[4] = 800.0
    z_t = RNG.normal(0, 1, 9)
    assert O.token_kl(z_s, z_t) == pytest.approx(-scipy.special.log_softmax(z_t)[4], rel=1e-12)


def test_sampled_cost_sign_and_expectation():
    z_s = np.log([0.5, 0.5]); z_t = np.log([0.25, 0.75])
    assert O.token_cost(z_s, z_t, 0) == pytest.approx(math.log(2.0), rel=1e-13)
    assert O.token_cost(z_s, z_t, 1) == pytest.approx(math.log(0.5 / 0.75), rel=1e-13)
    V = 11
    z_s, z_t = RNG.normal(0, 2, V), RNG.normal(0, 2, V)
    p = scipy.special.softmax(z_s)
    exp_c = sum(p[y] * O.token_cost(z_s, z_t, y) for y in range(V))
    assert exp_c == pytest.approx(O.token_kl(z_s, z_t), rel=1e-12)
    # Monte-Carlo: the mean of sampled costs approaches the full-vocabulary KL
    ys = np.random.default_rng(3).choice(V, size=200000, p=p)
    costs = np.array([O.token_cost(z_s, z_t, y) for y in range(V)])
    assert costs[ys].mean() == pytest.approx(O.token_kl(z_s, z_t), abs=0.02)


# ---------------------------------------------------------------- gradients

@pytest.mark.parametrize("V", [2, 7, 16])
def test_dz_finite_differences_and_row_sum(V):
    z_s, z_t = RNG.normal(0, 2, V), RNG.normal(0, 2, V)
    dz = O.token_dz(z_s, z_t)
    assert abs(dz.sum()) < 1e-15
    eps = 1e-6
    for v in range(V):
        e = np.zeros(V); e[v] = eps
        fd = (O.token_kl(z_s + e, z_t) - O.token_kl(z_s - e, z_t)) / (2 * eps)
        assert dz[v] == pytest.approx(fd, rel=1e-6, abs=1e-9)
    # teacher is frozen: a teacher perturbation must not be what dz differentiates
    fd_t = (O.token_kl(z_s, z_t + e) - O.token_kl(z_s, z_t - e)) / (2 * eps)
    assert abs(fd_t - dz[V - 1]) > 1e-4
    assert np.all(O.token_dz(z_s, z_s) == 0.0)


def test_dz_is_expected_sampled_token_gradient():
    # Eq. 4 at one position, in logit space: c_t * d log p_s(y) / d z_s = c_t (e_y - p_s);
    # its expectation over y ~ p_s, by exhaustive enumeration.
    V = 9
    z_s, z_t = RNG.normal(0, 2, V), RNG.normal(0, 2, V)
    p = scipy.special.softmax(z_s)
    acc = np.zeros(V)
    for y in range(V):
        c = scipy.special.log_softmax(z_s)[y] - scipy.special.log_softmax(z_t)[y]
        acc += p[y] * c * (np.eye(V)[y] - p)
    assert np.allclose(O.token_dz(z_s, z_t), acc, rtol=1e-12, atol=1e-15)


def test_sampled_estimator_gradient():
    # Eq. 4 at one position: c_t held fixed multiplies the score of the sampled token
    V = 11
    z_s, z_t = RNG.normal(0, 2, V), RNG.normal(0, 2, V)
    p = scipy.special.softmax(z_s)
    for y in (0, 4, V - 1):
        dz = O.token_dz_sampled(z_s, z_t, y)
        c = scipy.special.log_softmax(z_s)[y] - scipy.special.log_softmax(z_t)[y]
        assert abs(dz.sum()) < 1e-12                       # a score: sums to zero
        eps = 1e-6                                          # finite differences of c * log p_s(y)
        for v in range(V):
            e = np.zeros(V); e[v] = eps
            fd = c * (scipy.special.log_softmax(z_s + e)[y] - scipy.special.log_softmax(z_s - e)[y]) / (2 * eps)
            assert dz[v] == pytest.approx(fd, rel=1e-6, abs=1e-9)
    # its expectation over y ~ p_s is the gradient of the full-vocabulary KL
    acc = sum(p[y] * O.token_dz_sampled(z_s, z_t, y) for y in range(V))
    assert np.allclose(acc, O.token_dz(z_s, z_t), rtol=1e-12, atol=1e-15)
    # teacher == student: c_t = 0, no update
    assert not O.token_dz_sampled(z_s, z_s, 3).any()
    # through the hidden state: g = dz W_s, and the batched path agrees with the single row
    Hs, Ht = 5, 4
    W_s, W_t = RNG.normal(0, 0.7, (V, Hs)), RNG.normal(0, 0.7, (V, Ht))
    H_s, H_t = RNG.normal(0, 1, (3, Hs)), RNG.normal(0, 1, (3, Ht))
    ids = np.array([2, 7, 0])
    _, c, g = O.rows_terms(H_s, H_t, W_s, W_t, ids, estimator=O.EST_SAMPLED)
    for r in range(3):
        pr = scipy.special.softmax(W_s @ H_s[r])
        want = c[r] * (W_s[ids[r]] - pr @ W_s)
        assert np.allclose(g[r], want, rtol=1e-12, atol=1e-15)
        assert np.allclose(g[r], O.token_terms(H_s[r], H_t[r], W_s, W_t, int(ids[r]), O.EST_SAMPLED)[2],
                           rtol=1e-12, atol=1e-15)


def test_hidden_gradient_finite_differences_and_layout():
    V, Hs, Ht = 13, 5, 4
    W_s, W_t = RNG.normal(0, 0.7, (V, Hs)), RNG.normal(0, 0.7, (V, Ht))
    h_s, h_t = RNG.normal(0, 1, Hs), RNG.normal(0, 1, Ht)
    kl, c, g = O.token_terms(h_s, h_t, W_s, W_t, 3)
    # layout: z[v] = sum_k h[k] W[v,k], written out with loops
    z_s = np.array([sum(h_s[k] * W_s[v, k] for k in range(Hs)) for v in range(V)])
    z_t = np.array([sum(h_t[k] * W_t[v, k] for k in range(Ht)) for v in range(V)])
    assert kl == pytest.approx(scipy.stats.entropy(scipy.special.softmax(z_s),
                                                   scipy.special.softmax(z_t)), rel=1e-12)
    assert c == pytest.approx(scipy.special.log_softmax(z_s)[3]
                              - scipy.special.log_softmax(z_t)[3], rel=1e-12)
    eps = 1e-6
    for k in range(Hs):
        e = np.zeros(Hs); e[k] = eps
        fd = (O.token_terms(h_s + e, h_t, W_s, W_t)[0]
              - O.token_terms(h_s - e, h_t, W_s, W_t)[0]) / (2 * eps)
        assert g[k] == pytest.approx(fd, rel=1e-6, abs=1e-9)
    # batched rows equal the single-row definition
    Hs_rows, Ht_rows = RNG.normal(0, 1, (37, Hs)), RNG.normal(0, 1, (37, Ht))
    ids = RNG.integers(0, V, 37)
    kls, cs, gs = O.rows_terms(Hs_rows, Ht_rows, W_s, W_t, ids, block=8)
    for r in (0, 7, 8, 36):
        k1, c1, g1 = O.token_terms(Hs_rows[r], Ht_rows[r], W_s, W_t, int(ids[r]))
        assert kls[r] == pytest.approx(k1, rel=1e-12)
        assert cs[r] == pytest.approx(c1, rel=1e-12)
        assert np.allclose(gs[r], g1, rtol=1e-12, atol=1e-16)


# ---------------------------------------------------------------- windows and alignment

def _small_problem(seed=0, B=4, V=23, Hs=6, Ht=5):
    g = np.random.default_rng(seed)
    lens = g.integers(1, 9, size=B)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    T = int(offsets[-1])
    return dict(h_s=g.normal(0, 1, (T, Hs)), h_t=g.normal(0, 1, (T, Ht)),
                W_s=g.normal(0, 0.5, (V, Hs)), W_t=g.normal(0, 0.5, (V, Ht)),
                ids=g.integers(0, V, T), offsets=offsets), lens


def test_window_covering_rollout_gives_full_loss_and_unit_alignment():
    pr, lens = _small_problem(1)
    out = O.supervise(**pr, window=lens + 3, mode=O.MODE_PREFIX_AND_FULL)
    assert np.array_equal(out["loss_prefix"], out["loss_full"])        # bit for bit
    assert np.array_equal(out["dh_prefix"], out["dh_full"])
    assert np.allclose(out["rho_pooled"], 1.0, atol=1e-12)
    assert np.allclose(out["rho_field"], 1.0, atol=1e-12)
    assert np.allclose(out["batch"][2:6], 1.0, atol=1e-12)
    assert out["batch"][0] == out["batch"][1]


def test_prefix_rows_are_a_subset_of_full_rows_and_rest_is_zero():
    pr, lens = _small_problem(2)
    window = np.maximum(lens // 2, 1)
    full = O.supervise(**pr, window=window, mode=O.MODE_PREFIX_AND_FULL, reduction=O.RED_SUM)
    pre = O.supervise(**pr, window=window, mode=O.MODE_PREFIX_ONLY, reduction=O.RED_SUM)
    adm = O.plan(pr["offsets"], window)["rows"]
    mask = np.zeros(len(full["kl"]), bool); mask[adm] = True
    assert np.array_equal(pre["kl"][mask], full["kl"][mask])
    assert np.array_equal(pre["dh_prefix"], full["dh_prefix"])
    assert np.all(pre["kl"][~mask] == 0) and np.all(pre["dh_prefix"][~mask] == 0)
    assert np.all(pre["loss_full"] == 0) and np.all(pre["rho_pooled"] == 0)
    # per-window loss is the token mean over exactly n_i rows
    for i in range(len(lens)):
        o = int(pr["offsets"][i])
        assert full["loss_prefix"][i] == pytest.approx(full["kl"][o:o + window[i]].mean(), rel=1e-13)
        assert full["loss_full"][i] == pytest.approx(full["kl"][o:o + lens[i]].mean(), rel=1e-13)


def test_reductions_and_grad_scale():
    pr, lens = _small_problem(3)
    window = np.array([2, 1, 100, 3])[: len(lens)]
    n = np.minimum(window, lens)
    B = len(lens)
    outs = {r: O.supervise(**pr, window=window, mode=O.MODE_PREFIX_AND_FULL, reduction=r)
            for r in (O.RED_SEQ_MEAN, O.RED_SUM, O.RED_TOKEN_MEAN)}
    kl = outs[O.RED_SUM]["kl"]
    adm = O.plan(pr["offsets"], window)["rows"]
    assert outs[O.RED_SUM]["batch"][0] == pytest.approx(kl[adm].sum(), rel=1e-13)
    assert outs[O.RED_SUM]["batch"][1] == pytest.approx(kl.sum(), rel=1e-13)
    assert outs[O.RED_TOKEN_MEAN]["batch"][0] == pytest.approx(kl[adm].mean(), rel=1e-13)
    assert outs[O.RED_TOKEN_MEAN]["batch"][1] == pytest.approx(kl.mean(), rel=1e-13)
    assert outs[O.RED_SEQ_MEAN]["batch"][0] == pytest.approx(outs[O.RED_SEQ_MEAN]["loss_prefix"].mean(), rel=1e-13)
    assert outs[O.RED_SEQ_MEAN]["batch"][1] == pytest.approx(outs[O.RED_SEQ_MEAN]["loss_full"].mean(), rel=1e-13)
    # dh is the gradient of the batch objective: seq-mean weights are 1/(B n_i), 1/(B len_i)
    g = outs[O.RED_SUM]["g"]
    for i in range(B):
        o = int(pr["offsets"][i])
        assert np.allclose(outs[O.RED_SEQ_MEAN]["dh_prefix"][o], g[o] / (B * n[i]), rtol=1e-13)
        assert np.allclose(outs[O.RED_SEQ_MEAN]["dh_full"][o], g[o] / (B * lens[i]), rtol=1e-13)
    # per-rollout alignment does not depend on the reduction; the gradient is linear in grad_scale
    for r in outs:
        assert np.allclose(outs[r]["rho_pooled"], outs[O.RED_SUM]["rho_pooled"], atol=1e-12)
        assert np.allclose(outs[r]["rho_field"], outs[O.RED_SUM]["rho_field"], atol=1e-12)
    s = O.supervise(**pr, window=window, mode=O.MODE_PREFIX_AND_FULL, grad_scale=-2.5)
    assert np.allclose(s["dh_prefix"], -2.5 * outs[O.RED_SEQ_MEAN]["dh_prefix"], rtol=1e-13)
    assert np.allclose(s["rho_pooled"], outs[O.RED_SEQ_MEAN]["rho_pooled"], atol=1e-12)


def test_batch_objective_gradient_by_finite_differences():
    # dh_prefix must be the derivative of batch[0] with respect to h_s, dh_full of batch[1].
    pr, lens = _small_problem(4, B=3, V=11, Hs=4, Ht=3)
    window = np.array([1, 3, 2])
    out = O.supervise(**pr, window=window, mode=O.MODE_PREFIX_AND_FULL)
    eps = 1e-6
    for (t, k) in [(0, 0), (int(pr["offsets"][1]) + 1, 2), (int(pr["offsets"][2]), 3),
                   (int(pr["offsets"][3]) - 1, 1)]:
        hp, hm = pr["h_s"].copy(), pr["h_s"].copy()
        hp[t, k] += eps; hm[t, k] -= eps
        bp = O.supervise(**{**pr, "h_s": hp}, window=window, mode=O.MODE_PREFIX_AND_FULL)["batch"]
        bm = O.supervise(**{**pr, "h_s": hm}, window=window, mode=O.MODE_PREFIX_AND_FULL)["batch"]
        assert out["dh_prefix"][t, k] == pytest.approx((bp[0] - bm[0]) / (2 * eps), rel=1e-5, abs=1e-10)
        assert out["dh_full"][t, k] == pytest.approx((bp[1] - bm[1]) / (2 * eps), rel=1e-5, abs=1e-10)


def test_permutation_and_concatenation_invariance():
    pr, lens = _small_problem(5, B=5)
    window = np.array([2, 9, 1, 3, 4])
    base = O.supervise(**pr, window=window, mode=O.MODE_PREFIX_AND_FULL, reduction=O.RED_SUM)
    perm = [3, 0, 4, 1, 2]
    rows = np.concatenate([np.arange(pr["offsets"][i], pr["offsets"][i + 1]) for i in perm])
    pr2 = dict(pr, h_s=pr["h_s"][rows], h_t=pr["h_t"][rows], ids=pr["ids"][rows],
               offsets=np.concatenate([[0], np.cumsum(lens[perm])]))
    out2 = O.supervise(**pr2, window=window[perm], mode=O.MODE_PREFIX_AND_FULL, reduction=O.RED_SUM)
    for key in ("loss_prefix", "loss_full", "rho_pooled", "rho_field"):
        assert np.allclose(out2[key], base[key][perm], rtol=1e-13, atol=1e-15)
    # the first two rollouts alone give the same per-rollout numbers
    cut = int(pr["offsets"][2])
    pr3 = dict(pr, h_s=pr["h_s"][:cut], h_t=pr["h_t"][:cut], ids=pr["ids"][:cut],
               offsets=pr["offsets"][:3])
    out3 = O.supervise(**pr3, window=window[:2], mode=O.MODE_PREFIX_AND_FULL, reduction=O.RED_SUM)
    for key in ("loss_prefix", "loss_full", "rho_pooled", "rho_field"):
        assert np.allclose(out3[key], base[key][:2], rtol=1e-13, atol=1e-15)
    assert np.allclose(out3["dh_prefix"], base["dh_prefix"][:cut], rtol=1e-13, atol=1e-18)


def test_alignment_hand_built_gradients():
    H = 4
    e = np.eye(H)
    # one rollout of 7 rows, window 3: prefix rows e1, suffix rows e2 -> cos = 3/5
    g = np.stack([e[0]] * 3 + [e[1]] * 4)
    for red in (O.RED_SEQ_MEAN, O.RED_SUM, O.RED_TOKEN_MEAN):
        out = O.window_outputs(np.zeros(7), g, [0, 7], [3], red)
        assert out["rho_pooled"][0] == pytest.approx(0.6, abs=1e-14)
        assert out["rho_field"][0] == pytest.approx(math.sqrt(3 / 7), abs=1e-14)
    # suffix opposite and stronger than the prefix -> cos = -1 pooled
    g = np.stack([e[0]] * 3 + [-e[0]] * 4)
    out = O.window_outputs(np.zeros(7), g, [0, 7], [3])
    assert out["rho_pooled"][0] == pytest.approx(-1.0, abs=1e-14)
    assert out["rho_field"][0] == pytest.approx(math.sqrt(3 / 7), abs=1e-14)
    # two rollouts whose suffix noise cancels after batch aggregation: micro = 1 > macro = 0.6
    g = np.stack([e[0]] * 3 + [e[1]] * 4 + [e[0]] * 3 + [-e[1]] * 4)
    out = O.window_outputs(np.zeros(14), g, [0, 7, 14], [3, 3])
    assert np.allclose(out["rho_pooled"], 0.6, atol=1e-14)
    assert out["batch"][4] == pytest.approx(0.6, abs=1e-14)
    assert out["batch"][2] == pytest.approx(1.0, abs=1e-14)
    # empty window / empty rollout: alignment 0 and left out of the macro mean
    out = O.window_outputs(np.zeros(14), g, [0, 7, 7, 14], [3, 5, 0])
    assert out["rho_pooled"].tolist() == pytest.approx([0.6, 0.0, 0.0])
    assert out["batch"][4] == pytest.approx(0.6, abs=1e-14)
    assert np.all(np.abs(out["rho_pooled"]) <= 1.0)


def test_field_alignment_closed_form_random():
    pr, lens = _small_problem(6, B=4)
    window = np.array([1, 2, 3, 1])
    out = O.supervise(**pr, window=window, mode=O.MODE_PREFIX_AND_FULL)
    n = np.minimum(window, lens)
    for i in range(4):
        o = int(pr["offsets"][i])
        S_n = (out["g"][o:o + n[i]] ** 2).sum()
        S_l = (out["g"][o:o + lens[i]] ** 2).sum()
        assert out["rho_field"][i] == pytest.approx(math.sqrt(S_n / S_l), rel=1e-12)
        assert -1 - 1e-12 <= out["rho_pooled"][i] <= 1 + 1e-12


def test_field_micro_cosine_closed_form_with_unequal_weights():
    """batch[3], the cosine of the two whole [T, H_s] gradient arrays (Sec. 4.2's cosine after
    batch aggregation, Fig. 5 "micro", in the field reading): with S_i(m) the sum of squared row
    norms of g over the first m rows of rollout i it is
    sum_i a^p_i a^f_i S_i(n_i) / sqrt(sum_i a^p_i^2 S_i(n_i) * sum_i a^f_i^2 S_i(len_i)).
    Rollouts of different lengths and windows give unequal weights, so it differs from the pooled
    micro cosine, from the macro mean and from any unweighted version."""
    pr, lens = _small_problem(12, B=5)
    window = np.array([1, 3, 2, 100, 1])
    n = np.minimum(window, lens)
    for red in (O.RED_SEQ_MEAN, O.RED_TOKEN_MEAN, O.RED_SUM):
        out = O.supervise(**pr, window=window, mode=O.MODE_PREFIX_AND_FULL, reduction=red, grad_scale=0.7)
        B = len(lens)
        if red == O.RED_SEQ_MEAN:
            ap, af = 1.0 / (B * n), 1.0 / (B * lens)
        elif red == O.RED_TOKEN_MEAN:
            ap, af = np.full(B, 1.0 / n.sum()), np.full(B, 1.0 / lens.sum())
        else:
            ap = af = np.ones(B)
        S_n = np.array([(out["g"][pr["offsets"][i]:pr["offsets"][i] + n[i]] ** 2).sum() for i in range(B)])
        S_l = np.array([(out["g"][pr["offsets"][i]:pr["offsets"][i + 1]] ** 2).sum() for i in range(B)])
        want = (ap * af * S_n).sum() / math.sqrt((ap ** 2 * S_n).sum() * (af ** 2 * S_l).sum())
        assert out["batch"][3] == pytest.approx(want, rel=1e-12)
        # and it is none of its neighbours
        assert abs(out["batch"][3] - out["batch"][2]) > 1e-3      # pooled micro
        assert abs(out["batch"][3] - out["batch"][5]) > 1e-4      # field macro
    # the candidate audit's micro field cosine is the same quantity at a shared window
    a = O.audit_candidates(out["g"], pr["offsets"], (2,), O.RED_SEQ_MEAN)
    n2 = np.minimum(2, lens)
    S_2 = np.array([(out["g"][pr["offsets"][i]:pr["offsets"][i] + n2[i]] ** 2).sum() for i in range(len(lens))])
    ap2, af2 = 1.0 / (len(lens) * n2), 1.0 / (len(lens) * lens)
    want = (ap2 * af2 * S_2).sum() / math.sqrt((ap2 ** 2 * S_2).sum() * (af2 ** 2 * S_l).sum())
    assert a["micro_field"][0] == pytest.approx(want, rel=1e-12)


def test_macro_means_leave_out_rollouts_without_a_gradient():
    """Reading of Sec. 4.2 / Fig. 5 "macro": the mean of the per-rollout cosines over the rollouts
    whose two gradients are both non-zero.  Hand-built batch: rollout 0 regular, rollout 1 empty,
    rollout 2 with window 0, rollout 3 whose gradient rows are all zero."""
    H = 3
    e = np.eye(H)
    g = np.stack([e[0], e[1], e[1],            # rollout 0: len 3, window 1 -> field sqrt(1/3), pooled 1/sqrt(5)
                  e[2], e[2],                  # rollout 2: len 2, window 0
                  0 * e[0], 0 * e[0]])         # rollout 3: len 2, window 1, zero gradient
    offsets = [0, 3, 3, 5, 7]
    out = O.window_outputs(np.zeros(7), g, offsets, [1, 4, 0, 1])
    assert out["rho_field"].tolist() == pytest.approx([math.sqrt(1 / 3), 0.0, 0.0, 0.0])
    assert out["rho_pooled"].tolist() == pytest.approx([1 / math.sqrt(5), 0.0, 0.0, 0.0])
    assert out["batch"][5] == pytest.approx(math.sqrt(1 / 3), rel=1e-12)     # not sqrt(1/3) / 4
    assert out["batch"][4] == pytest.approx(1 / math.sqrt(5), rel=1e-12)
    # a second regular rollout enters both means with weight 1/2
    g2 = np.concatenate([g, np.stack([e[0], e[0], e[0], e[0]])])
    out = O.window_outputs(np.zeros(11), g2, offsets + [11], [1, 4, 0, 1, 1])
    assert out["batch"][5] == pytest.approx((math.sqrt(1 / 3) + 0.5) / 2, rel=1e-12)
    assert out["batch"][4] == pytest.approx((1 / math.sqrt(5) + 1.0) / 2, rel=1e-12)


def test_logits_given_sampled_estimator_agrees_with_hidden_state_path():
    """Eq. 4 on the sampled token through the logits-given variant: dz[t] = grad_scale a^p_i c_t
    (e_{y_t} - p_s), so dz W_s must be the dh_prefix of the hidden-state path under the same
    estimator, weights included (sequence-mean reduction, grad_scale != 1)."""
    pr, lens = _small_problem(13, B=4)
    window = np.array([2, 1, 5, 3])
    z_s, z_t = pr["h_s"] @ pr["W_s"].T, pr["h_t"] @ pr["W_t"].T
    a = O.supervise(**pr, window=window, mode=O.MODE_PREFIX_ONLY, reduction=O.RED_SEQ_MEAN,
                    grad_scale=-1.75, estimator=O.EST_SAMPLED)
    b = O.supervise_from_logits(z_s, z_t, pr["ids"], pr["offsets"], window, reduction=O.RED_SEQ_MEAN,
                                grad_scale=-1.75, estimator=O.EST_SAMPLED)
    assert np.abs(a["dh_prefix"]).max() > 1e-3
    assert np.allclose(b["dz"] @ pr["W_s"], a["dh_prefix"], rtol=1e-10, atol=1e-15)
    assert np.allclose(a["kl"], b["kl"], rtol=1e-12) and np.allclose(a["c"], b["c"], rtol=1e-12)
    # row by row: the weight is that of the row's own rollout, the score that of its own token
    n = np.minimum(window, lens)
    for i in range(4):
        for j in range(int(lens[i])):
            t = int(pr["offsets"][i]) + j
            if j < n[i]:
                p = scipy.special.softmax(z_s[t])
                c = scipy.special.log_softmax(z_s[t])[pr["ids"][t]] - scipy.special.log_softmax(z_t[t])[pr["ids"][t]]
                want = -1.75 / (4 * n[i]) * c * (np.eye(len(p))[pr["ids"][t]] - p)
                assert np.allclose(b["dz"][t], want, rtol=1e-11, atol=1e-16)
            else:
                assert not b["dz"][t].any()
    # the expected-gradient variant is a different array
    e = O.supervise_from_logits(z_s, z_t, pr["ids"], pr["offsets"], window, reduction=O.RED_SEQ_MEAN,
                                grad_scale=-1.75)
    assert np.abs(e["dz"] - b["dz"]).max() > 1e-3


def test_logits_given_variant_agrees_with_hidden_state_path():
    pr, lens = _small_problem(8, B=3)
    window = np.array([2, 1, 4])
    z_s, z_t = pr["h_s"] @ pr["W_s"].T, pr["h_t"] @ pr["W_t"].T
    a = O.supervise(**pr, window=window, mode=O.MODE_PREFIX_ONLY, grad_scale=3.0)
    b = O.supervise_from_logits(z_s, z_t, pr["ids"], pr["offsets"], window, grad_scale=3.0)
    assert np.allclose(a["kl"], b["kl"], rtol=1e-12) and np.allclose(a["c"], b["c"], rtol=1e-12)
    assert np.allclose(b["dz"] @ pr["W_s"], a["dh_prefix"], rtol=1e-11, atol=1e-16)
    assert np.allclose(a["loss_prefix"], b["loss_prefix"], rtol=1e-12)
    assert a["batch"][0] == pytest.approx(b["batch"][0], rel=1e-12)
    assert np.all(np.abs(b["dz"].sum(axis=1)) < 1e-14)


# ---------------------------------------------------------------- audit, scheduler, diagnostics

def _golden():
    vals = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = v.split()
    return vals


def test_paper_constants():
    gold = _golden()
    assert round(float(O.RHO_STAR), 3) == float(gold["rho_star"][0])
    assert O.snr(O.RHO_STAR) == pytest.approx(float(gold["snr_at_rho_star"][0]), rel=1e-12)
    assert list(O.CANDIDATE_WINDOWS) == [int(x) for x in gold["candidate_windows"]]


def test_scheduler_picks_shortest_admissible_window():
    cands = (64, 128, 256, 512)
    assert O.next_window([0.2, 0.71, 0.9, 0.95], cands) == 128
    assert O.next_window([0.8, 0.1, 0.9, 0.95], cands) == 64
    assert O.next_window([0.2, 0.3, 0.5, 0.70], cands) == 512      # none admissible: longest
    assert O.next_window([0.2, 0.3, O.RHO_STAR, 0.9], cands) == 256  # threshold is inclusive
    assert O.next_window([0.9, 0.2], (512, 64)) == 512


def test_audit_candidates_consistent_with_single_window():
    g_ = np.random.default_rng(9)
    lens = np.array([5, 9, 3])
    offsets = np.concatenate([[0], np.cumsum(lens)])
    g = g_.normal(0, 1, (int(offsets[-1]), 6))
    cands = (1, 2, 4, 16)
    a = O.audit_candidates(g, offsets, cands)
    for k, L in enumerate(cands):
        out = O.window_outputs(np.zeros(len(g)), g, offsets, [L] * 3)
        assert np.array_equal(a["rho_pooled"][k], out["rho_pooled"])
        assert a["micro"][k] == out["batch"][2] and a["macro"][k] == out["batch"][4]
    assert np.allclose(a["rho_pooled"][-1], 1.0, atol=1e-12) and a["micro"][-1] == pytest.approx(1.0)
    # pooled cosine by hand for L=2 on rollout 0 (seq-mean weights cancel in a cosine)
    up, uf = g[0:2].sum(0), g[0:5].sum(0)
    assert a["rho_pooled"][1][0] == pytest.approx(up @ uf / np.linalg.norm(up) / np.linalg.norm(uf), rel=1e-12)


def test_audit_field_cosine_closed_form():
    # the field cosine of a prefix with the whole rollout is sqrt(S(n) / S(len)), S = sum of
    # squared row norms, whatever the weights; written here without the oracle's code path
    g_ = np.random.default_rng(10)
    lens = np.array([7, 2, 11])
    offsets = np.concatenate([[0], np.cumsum(lens)])
    g = g_.normal(0, 1, (int(offsets[-1]), 5))
    cands = (1, 3, 8, 64)
    for red in (O.RED_SEQ_MEAN, O.RED_SUM, O.RED_TOKEN_MEAN):
        a = O.audit_candidates(g, offsets, cands, red)
        for k, L in enumerate(cands):
            for i in range(3):
                rows = g[offsets[i]:offsets[i + 1]]
                n = min(L, len(rows))
                want = math.sqrt((rows[:n] ** 2).sum() / (rows ** 2).sum())
                assert a["rho_field"][k][i] == pytest.approx(want, rel=1e-12)
        assert np.allclose(a["rho_field"][-1], 1.0) and a["micro_field"][-1] == pytest.approx(1.0)
        assert np.all(a["macro_field"] == pytest.approx(a["rho_field"].mean(axis=1)))


def test_head_weight_gradient_finite_differences():
    # dW = gradient of the batch objective with respect to the student LM-head weights
    V, Hs, Ht = 7, 4, 3
    W_s, W_t = RNG.normal(0, 0.7, (V, Hs)), RNG.normal(0, 0.7, (V, Ht))
    lens = np.array([3, 5])
    offsets = np.concatenate([[0], np.cumsum(lens)])
    T = int(offsets[-1])
    h_s, h_t = RNG.normal(0, 1, (T, Hs)), RNG.normal(0, 1, (T, Ht))
    window = np.array([2, 9])
    for red in (O.RED_SEQ_MEAN, O.RED_SUM, O.RED_TOKEN_MEAN):
        out = O.supervise(h_s, h_t, W_s, W_t, None, offsets, window, reduction=red, grad_scale=1.5,
                          mode=O.MODE_PREFIX_AND_FULL, head_gradient=True)

        def objectives(W):
            o = O.supervise(h_s, h_t, W, W_t, None, offsets, window, reduction=red,
                            mode=O.MODE_PREFIX_AND_FULL)
            return o["batch"][0], o["batch"][1]
        eps = 1e-6
        for v, k in ((0, 0), (3, 2), (6, 3)):
            E = np.zeros_like(W_s); E[v, k] = eps
            (pp, fp), (pm, fm) = objectives(W_s + E), objectives(W_s - E)
            assert out["dW_prefix"][v, k] == pytest.approx(1.5 * (pp - pm) / (2 * eps), rel=1e-6, abs=1e-9)
            assert out["dW_full"][v, k] == pytest.approx(1.5 * (fp - fm) / (2 * eps), rel=1e-6, abs=1e-9)
        assert np.allclose(out["dW_prefix"].sum(axis=0), 0, atol=1e-12)      # rows of dz sum to zero
    # consistent with the hidden-state gradient: both are contractions of the same dz
    out = O.supervise(h_s, h_t, W_s, W_t, None, offsets, window, reduction=O.RED_SUM,
                      mode=O.MODE_PREFIX_AND_FULL, head_gradient=True)
    x = RNG.normal(0, 1, V)       # x^T dW_full = sum_t (x . dz_t) h_s[t]; check through dz directly
    dz = np.stack([O.token_dz(W_s @ h_s[t], W_t @ h_t[t]) for t in range(T)])
    assert np.allclose(x @ out["dW_full"], (dz @ x) @ h_s, rtol=1e-12)
    same = O.supervise(h_s, h_s, W_s, W_s, None, offsets, window, mode=O.MODE_PREFIX_AND_FULL,
                       head_gradient=True)
    assert np.abs(same["dW_full"]).max() < 1e-15
    one = O.supervise(h_s, h_t, W_s, W_t, None, offsets, np.array([1, 0]), reduction=O.RED_SUM,
                      head_gradient=True)
    assert np.allclose(one["dW_prefix"], np.outer(dz[0], h_s[0]), rtol=1e-12)      # one admitted token


def test_teacher_diagnostics():
    assert O.teacher_branching_factor(np.zeros(37)) == pytest.approx(37.0, rel=1e-12)
    z = np.array([0.0, 50.0, 0.0])
    assert O.teacher_branching_factor(z) == pytest.approx(1.0, abs=1e-12)
    z = np.array([0.3, 2.0, -1.0, 2.0, 0.5])
    assert [O.teacher_rank(z, y) for y in range(5)] == [4, 1, 5, 1, 3]
    p = scipy.special.softmax(z)
    assert O.teacher_branching_factor(z) == pytest.approx(math.exp(scipy.stats.entropy(p)), rel=1e-12)
    assert O.teacher_entropy(np.zeros(37)) == pytest.approx(math.log(37.0), rel=1e-12)
    assert O.teacher_entropy(z) == pytest.approx(scipy.stats.entropy(p), rel=1e-12)
    assert O.teacher_entropy(z) == pytest.approx(math.log(O.teacher_branching_factor(z)), rel=1e-12)
    assert O.teacher_logp(z, 2) == pytest.approx(math.log(p[2]), rel=1e-12)
    assert O.teacher_logp(np.zeros(8), 3) == pytest.approx(-math.log(8.0), rel=1e-12)
    ranks = [[1, 2, 9, 1], [1, 1, 1, 1], [5, 1, 1, 1]]
    assert O.topk_survival(ranks, 3, 2) == pytest.approx(2 / 3)
    assert O.topk_survival(ranks, 3, 4) == pytest.approx(1 / 3)
    assert O.topk_survival(ranks, 10, 4) == 1.0


def test_rollout_summaries_of_the_diagnostics():
    # first rejection <-> survival fraction: S_T^(k) = share of rollouts whose first rejection is >= T
    g = np.random.default_rng(11)
    ranks = [list(g.integers(1, 9, size=int(n))) for n in (5, 1, 9, 0, 7, 12)]
    for k in (1, 3, 5, 8):
        fr = [O.first_rejection(r, k) for r in ranks]
        for T in range(0, 13):
            assert O.topk_survival(ranks, k, T) == pytest.approx(np.mean([f >= min(T, len(r)) for f, r in zip(fr, ranks)]))
    assert O.first_rejection([1, 2, 7, 1], 3) == 2 and O.first_rejection([1, 2, 3], 3) == 3
    assert O.first_rejection([], 3) == 0 and O.first_rejection([9], 3) == 0
    # region means: hand example, empty regions, batch row weighted by tokens
    offsets = np.array([0, 4, 4, 7])
    v = np.array([1.0, 3.0, 5.0, 7.0, 10.0, 20.0, 60.0])
    m = O.region_means(v, offsets, n=[1, 0, 3], computed=[4, 0, 3])
    assert np.allclose(m, [[1.0, 5.0], [0.0, 0.0], [30.0, 0.0], [(1 + 90) / 4, 5.0]])
    m = O.region_means(v, offsets, n=[1, 0, 3], computed=[1, 0, 3])       # prefix-only: no suffix anywhere
    assert np.allclose(m[:, 1], 0) and m[3, 0] == pytest.approx(91 / 4)
    # loss share: uniform loss -> share of positions; monotone; 1 at L >= longest; hand example
    lens = np.array([3, 10, 6]); off = np.concatenate([[0], np.cumsum(lens)])
    cands = [1, 2, 4, 8, 16]
    sh = O.loss_share(np.full(19, 0.25), off, lens, cands)
    assert np.allclose(sh, [np.minimum(L, lens).sum() / 19 for L in cands])
    kl = g.random(19)
    sh = O.loss_share(kl, off, lens, cands)
    assert np.all(np.diff(sh) >= 0) and sh[-1] == pytest.approx(1.0)
    assert sh[0] == pytest.approx((kl[0] + kl[3] + kl[13]) / kl.sum())
    assert not O.loss_share(np.zeros(19), off, lens, cands).any()
    sh = O.loss_share(kl, off, [2, 0, 6], [1, 4])                         # computed rows only
    assert sh[1] == pytest.approx((kl[0] + kl[1] + kl[13:17].sum()) / (kl[0] + kl[1] + kl[13:19].sum()))


def test_head_block_alignment():
    # rho_head = cos(dW_prefix, dW_full): pinned through the Gram identity
    # <dW_p, dW_f> = sum_{r, r'} w^p_r w^f_r' (dz_r . dz_r') (h_r . h_r'), never forming dW
    V, Hs, Ht = 9, 5, 4
    W_s, W_t = RNG.normal(0, 0.7, (V, Hs)), RNG.normal(0, 0.7, (V, Ht))
    lens = np.array([4, 6, 2]); offsets = np.concatenate([[0], np.cumsum(lens)]); T = int(offsets[-1])
    h_s, h_t = RNG.normal(0, 1, (T, Hs)), RNG.normal(0, 1, (T, Ht))
    window = np.array([2, 3, 0])
    out = O.supervise(h_s, h_t, W_s, W_t, None, offsets, window, reduction=O.RED_SEQ_MEAN, grad_scale=2.0,
                      mode=O.MODE_PREFIX_AND_FULL, head_gradient=True)
    dz = np.stack([O.token_dz(W_s @ h_s[t], W_t @ h_t[t]) for t in range(T)])
    ap, af = O.row_weights(lens, np.minimum(window, lens), O.RED_SEQ_MEAN)
    wp, wf = np.zeros(T), np.zeros(T)
    for i in range(3):
        o = offsets[i]
        wp[o:o + min(window[i], lens[i])] = ap[i]
        wf[o:o + lens[i]] = af[i]
    G = (dz @ dz.T) * (h_s @ h_s.T)
    want = (wp @ G @ wf) / math.sqrt((wp @ G @ wp) * (wf @ G @ wf))
    assert out["rho_head"] == pytest.approx(want, rel=1e-10)
    # the window covers everything -> the two objectives coincide
    full = O.supervise(h_s, h_t, W_s, W_t, None, offsets, lens + 3, mode=O.MODE_PREFIX_AND_FULL,
                       head_gradient=True)
    assert full["rho_head"] == pytest.approx(1.0, abs=1e-12)
    none = O.supervise(h_s, h_t, W_s, W_t, None, offsets, np.zeros(3, int), mode=O.MODE_PREFIX_AND_FULL,
                       head_gradient=True)
    assert none["rho_head"] == 0.0


def test_cosine_against_angles_and_the_zero_convention():
    """cos between plane vectors at known angles; scale invariance; a zero norm gives 0 (the
    convention the alignment outputs follow)."""
    for deg in (0.0, 30.0, 90.0, 135.0, 180.0):
        th = math.radians(deg)
        a, b = np.array([2.0, 0.0, 0.0]), 5.0 * np.array([math.cos(th), math.sin(th), 0.0])
        assert O.cosine(a, b) == pytest.approx(math.cos(th), abs=1e-15)
        assert O.cosine(-3.0 * a, b) == pytest.approx(-math.cos(th), abs=1e-15)
    assert O.cosine(np.zeros(4), np.ones(4)) == 0.0 and O.cosine(np.ones(4), np.zeros(4)) == 0.0
    m = RNG.normal(size=(3, 5))
    assert O.cosine(m, 2.0 * m) == pytest.approx(1.0)          # arrays are flattened
