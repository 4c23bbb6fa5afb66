"""Shared parity helpers: tolerances (stated once, used by every GPU parity test) and
conversion of the seeded inputs into what the oracle takes."""
import numpy as np

from paper_2605_28396_amd import synth
from tests import error_model

# Tolerances: bf16 inputs, fp32 accumulation on the GPU, fp64 oracle.
KL_REL = 1e-3          # |dKL| <= KL_REL * KL  (+ KL_ABS floor for tiny KL)
KL_ABS = 1e-6
C_REL = 1e-3           # |dc| <= C_REL * max(1, |c|)
DH_ABS = 2e-3          # max |d dh| <= DH_ABS  and  <= DH_REL * max|dh_oracle|
DH_REL = 2e-3
RHO_ABS = 2e-3
LOSS_REL = 1e-3
BF16_ULP = 2.0 ** -8   # storage rounding of a bf16 output element, relative
# Head-weight gradient dW[v][k] = sum_r w_r dz_r[v] h_s[r][k]: the kernels round the dz factor
# of every summand to bf16 three times (the two stored gradient factors, then w dz), each a
# relative error uniform in +-2^-9 at worst, rms 2^-9 / sqrt(3); the three together have rms
# 2^-9 and are independent across summands, so the error of an element has standard deviation
# <= 2^-9 * (Euclidean norm of its summands).  With few hundred rows the summands are heavy-
# tailed and an element can be one summand, so no fraction of max|dW| below 2^-8 is safe; the
# per-element bound is, and a dropped or misplaced row breaks it for most elements.
DW_SIGMA = 2.0 ** -9
DW_SIGMAS = 8.0        # max over ~1e6..1e9 elements of a sum of bounded errors stays below 6 sigma


def oracle_inputs(p: dict) -> dict:
    return {k: (v.cpu().numpy() if k == "ids" else synth.to_f64(v)) for k, v in p.items()}


def assert_kl(got, want, what="kl", logit_scale=None):
    """logit_scale: per-row magnitude of the logits (e.g. the larger |log-sum-exp|).  fp32
    logits of magnitude |z| carry an absolute rounding error of about 2^-24 |z| each, and the
    KL is a difference of such quantities: where the logits are tens of nats the absolute floor
    grows to 8 * 2^-24 * |z| (it is KL_ABS for |z| up to ~2)."""
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    err = np.abs(got - want)
    floor = KL_ABS if logit_scale is None else np.maximum(KL_ABS, 8 * 2.0 ** -24 * np.asarray(logit_scale))
    tol = KL_REL * np.abs(want) + floor
    bad = np.where(err > tol)[0]
    assert len(bad) == 0, f"{what}: {len(bad)} rows off, worst {err.max():.3e} at {bad[:5]}"


def assert_cost(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    err = np.abs(got - want)
    tol = C_REL * np.maximum(1.0, np.abs(want))
    assert np.all(err <= tol), f"c: worst {err.max():.3e}"


def assert_grad(got, want, what="dh", storage_ulp=0.0, abs_cap=True):
    """abs_cap: also hold the absolute bound DH_ABS, which is the binding one only while the
    gradients themselves are below 1 (the benchmark's random-initialisation regime); peaked
    cases with gradients of order 1..10 are held to the relative bound alone."""
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    scale = np.abs(want).max() if want.size else 0.0
    err = np.abs(got - want)
    tol = (np.minimum(DH_ABS, DH_REL * scale) if abs_cap else DH_REL * scale) + storage_ulp * np.abs(want)
    worst = (err - tol).max() if err.size else -1.0
    assert worst <= 0, (f"{what}: max err {err.max():.3e} vs tol {DH_REL * scale:.3e} "
                        f"(max|ref| {scale:.3e})")
    # rows that must be exactly zero are exactly zero
    zero_rows = ~np.any(want.reshape(want.shape[0], -1) != 0, axis=1)
    assert not np.any(got.reshape(got.shape[0], -1)[zero_rows] != 0), f"{what}: non-zero outside windows"


def assert_close_rel(got, want, rel, what):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    err = np.abs(got - want)
    assert np.all(err <= rel * np.abs(want) + 1e-7), f"{what}: worst {err.max():.3e}"


def summand_norms(f, w, rows, reduction, grad_scale=1.0, estimator=0, head=False, block=64):
    """Per-element error scales of the gradient outputs (tests/error_model.py) for workload w:
    g_l2 [T, H_s] for the unweighted row gradients and, with head, dW_prefix_l2 / dW_full_l2
    for the weighted head-weight gradients.  The weights are those of the reduction."""
    lens = np.diff(w.offsets)
    n = np.minimum(w.window.astype(np.int64), lens)
    B = len(n)
    if reduction == 0:        # sequence mean
        ap = np.where(n > 0, 1.0 / (B * np.maximum(n, 1)), 0.0)
        af = np.where(lens > 0, 1.0 / (B * np.maximum(lens, 1)), 0.0)
    elif reduction == 1:      # sum
        ap = af = np.ones(B)
    else:                     # token mean
        ap = np.full(B, 1.0 / n.sum() if n.sum() else 0.0)
        af = np.full(B, 1.0 / lens.sum() if lens.sum() else 0.0)
    return error_model.problem_norms(f, w.offsets, w.window, rows, ap, af, grad_scale, estimator, head, block)


def assert_grad_elementwise(got, want, l2, what="dh"):
    """Every element within DW_SIGMAS * 2^-9 of the Euclidean norm of its own summands (l2, already
    carrying the element's weight): the bound for gradients whose elements sum too few terms
    for a fraction of the largest element to mean anything."""
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    tol = DW_SIGMAS * DW_SIGMA * l2 + 1e-6 * (np.abs(want).max() if want.size else 0.0)
    err = np.abs(got - want)
    assert (err <= tol).all(), (what, err.max(), (err / np.maximum(tol, 1e-300)).max())
    zero_rows = ~np.any(want.reshape(want.shape[0], -1) != 0, axis=1)
    assert not np.any(got.reshape(got.shape[0], -1)[zero_rows] != 0), f"{what}: non-zero outside windows"
