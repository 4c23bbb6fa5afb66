"""Pins of the rounding-error model the GPU tests use for per-element bounds
(tests/error_model.py): closed forms on two entries, dominance over the gradient itself, and
the summand norms written out with loops."""
import math

import numpy as np
import pytest

from oracle import adwin_oracle as O
from tests import error_model as E

RNG = np.random.default_rng(11)


def test_error_scale_of_the_logit_gradient():
    # p (|Delta - KL| + D): two-entry closed form, dominance over |dz|, zero for equal models
    a, b = 0.8, 0.3                                   # p_s = (a, 1-a), p_t = (b, 1-b)
    z_s, z_t = np.log([a, 1 - a]), np.log([b, 1 - b])
    delta = np.array([math.log(a / b), math.log((1 - a) / (1 - b))])
    kl = a * delta[0] + (1 - a) * delta[1]
    dev = math.sqrt(a * (delta[0] - kl) ** 2 + (1 - a) * (delta[1] - kl) ** 2)
    want = np.array([a, 1 - a]) * (np.abs(delta - kl) + dev)
    assert np.allclose(E.dz_scale(z_s, z_t), want, rtol=1e-12)
    assert np.allclose(E.dz_scale(z_s + 3.0, z_t - 1.0), want, rtol=1e-12)     # shift invariance
    for _ in range(5):
        zs, zt = RNG.normal(0, 3, 11), RNG.normal(0, 3, 11)
        assert (E.dz_scale(zs, zt) >= np.abs(O.token_dz(zs, zt)) - 1e-15).all()
        assert np.abs(E.dz_scale(zs, zs + 2.5)).max() < 1e-12


def test_error_scale_of_the_sampled_gradient():
    zs, zt = RNG.normal(0, 3, 9), RNG.normal(0, 3, 9)
    for y in (0, 4, 8):
        sc, dz = E.dz_sampled_scale(zs, zt, y), O.token_dz_sampled(zs, zt, y)
        c = abs(O.token_cost(zs, zt, y))
        assert (sc >= np.abs(dz) * (1 - 1e-12) - 1e-15).all()
        assert sc[y] == pytest.approx(c) and sc.sum() == pytest.approx(c * (2 - np.exp(O.log_softmax(zs))[y]))


def test_summand_norms():
    V, Hs, Ht = 6, 3, 4
    W_s, W_t = RNG.normal(0, 0.7, (V, Hs)), RNG.normal(0, 0.7, (V, Ht))
    offsets = np.array([0, 3]); h_s, h_t = RNG.normal(0, 1, (3, Hs)), RNG.normal(0, 1, (3, Ht))
    f = dict(h_s=h_s, h_t=h_t, W_s=W_s, W_t=W_t, ids=None)
    out = O.supervise(h_s, h_t, W_s, W_t, None, offsets, np.array([2]), reduction=O.RED_SUM, head_gradient=True)
    nrm = E.problem_norms(f, offsets, np.array([2]), out["rows"], [1.0], [1.0], head=True)
    sc = np.stack([E.dz_scale(W_s @ h_s[t], W_t @ h_t[t]) for t in range(3)])
    for t in range(3):
        for k in range(Hs):
            terms = sc[t] * W_s[:, k]
            want = math.sqrt(sum(x * x for x in terms)) if t < 2 else 0.0
            assert nrm["g_l2"][t, k] == pytest.approx(want, rel=1e-12)
            if t < 2:
                assert abs(out["g"][t, k]) <= math.sqrt(V) * nrm["g_l2"][t, k] + 1e-15
    # head-weight summands: rows 0 and 1 carry weight 1 under the prefix objective
    for v in range(V):
        for k in range(Hs):
            want = math.sqrt(sum((sc[t, v] * h_s[t, k]) ** 2 for t in range(2)))
            assert nrm["dW_prefix_l2"][v, k] == pytest.approx(want, rel=1e-12)
    assert (np.abs(out["dW_prefix"]) <= math.sqrt(2) * nrm["dW_prefix_l2"] + 1e-15).all()
    # one admitted token: the norm is the summand itself
    one = E.problem_norms(f, offsets, np.array([1]), np.array([0]), [1.0], [1.0], head=True)
    assert np.allclose(one["dW_prefix_l2"], np.outer(sc[0], np.abs(h_s[0])), rtol=1e-12)
