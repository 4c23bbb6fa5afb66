"""GPU parity: the HIP path (called through the C ABI) against the fp64 oracle on the
same seeded inputs, element by element at sizes the oracle sweeps in seconds."""
import numpy as np
import pytest
import torch

from oracle import adwin_oracle as O
from paper_2605_28396_amd import synth
from tests import helpers as Hp

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2605_28396_amd import binding
    return binding


def _sample_ids_from_student(w, p):
    """Tiny config: ids drawn from the student's softmax by inverse CDF with seeded uniforms."""
    f = Hp.oracle_inputs(p)
    u = np.random.default_rng(synth.SEED).random(w.T)
    ids = np.zeros(w.T, np.int32)
    for t in range(w.T):
        ps = np.exp(O.log_softmax(f["W_s"] @ f["h_s"][t]))
        ids[t] = min(int(np.searchsorted(np.cumsum(ps), u[t])), w.V - 1)
    return torch.from_numpy(ids)


def _grad_l2(f, w, ref, reduction, grad_scale=1.0, estimator=0):
    """Per-element error scales of dh_prefix / dh_full: the summand norms of g times the weight
    of each row under the two objectives."""
    nrm = Hp.summand_norms(f, w, ref["rows"], reduction, grad_scale, estimator)["g_l2"]
    lens = np.diff(w.offsets)
    a_p, a_f = O.row_weights(lens, ref["n"], reduction)
    seq = np.repeat(np.arange(w.B), lens)
    adm = np.zeros(w.T, bool); adm[O.plan(w.offsets, w.window)["rows"]] = True
    wp = np.abs(grad_scale) * a_p[seq] * adm
    wf = np.abs(grad_scale) * a_f[seq]
    return nrm * wp[:, None], nrm * wf[:, None]


def _run_fused(B, w, p, dev, **kw):
    d = {k: v.to(dev) for k, v in p.items()}
    out = B.adwin_opd_fused(d["h_s"], d["h_t"], d["W_s"], d["W_t"], d["ids"], w.offsets, w.window,
                            mode=w.mode, **kw)
    torch.cuda.synchronize()
    return {k: v.float().cpu().numpy() if v.dtype.is_floating_point else v.cpu().numpy()
            for k, v in out.items()}


def _check_fused(w, got, ref, reduction, dh_bf16=False, logit_scale=None, abs_cap=True, grad_l2=None):
    """grad_l2: (l2 of dh_prefix, l2 of dh_full) -- hold the gradients to the per-element bound of
    their own summands (small vocabularies) instead of the fraction-of-maximum bar."""
    assert np.array_equal(got["n_out"], ref["n"]) and int(got["n_adm_out"][0]) == ref["n_adm"]
    assert int(got["status_dev"][0]) == 0
    Hp.assert_kl(got["kl"], ref["kl"], logit_scale=logit_scale)
    Hp.assert_cost(got["c"], ref["c"])
    ulp = Hp.BF16_ULP if dh_bf16 else 0.0
    probe = w.mode == synth.MODE_PREFIX_AND_FULL
    if grad_l2 is None:
        Hp.assert_grad(got["dh_prefix"], ref["dh_prefix"], "dh_prefix", ulp, abs_cap)
    else:
        Hp.assert_grad_elementwise(got["dh_prefix"], ref["dh_prefix"], grad_l2[0], "dh_prefix")
        if probe:
            Hp.assert_grad_elementwise(got["dh_full"], ref["dh_full"], grad_l2[1], "dh_full")
    Hp.assert_close_rel(got["loss_prefix"], ref["loss_prefix"], Hp.LOSS_REL, "loss_prefix")
    Hp.assert_close_rel(got["batch"][:2], ref["batch"][:2], Hp.LOSS_REL, "batch losses")
    if w.mode == synth.MODE_PREFIX_AND_FULL:
        if grad_l2 is None:
            Hp.assert_grad(got["dh_full"], ref["dh_full"], "dh_full", ulp, abs_cap)
        Hp.assert_close_rel(got["loss_full"], ref["loss_full"], Hp.LOSS_REL, "loss_full")
        for k in ("rho_pooled", "rho_field"):
            assert np.all(np.abs(got[k] - ref[k]) <= Hp.RHO_ABS), (k, got[k], ref[k])
        assert np.all(np.abs(got["batch"][2:6] - ref["batch"][2:6]) <= Hp.RHO_ABS), (got["batch"], ref["batch"])
    else:
        assert np.all(got["loss_full"] == 0) and np.all(got["rho_pooled"] == 0)
        assert np.all(got["batch"][1:] == 0)


@pytest.mark.parametrize("name,reduction", [
    ("tiny", O.RED_SUM), ("tiny", O.RED_SEQ_MEAN), ("tiny_probe", O.RED_SUM),
    ("tiny_probe", O.RED_SEQ_MEAN), ("tiny_probe", O.RED_TOKEN_MEAN),
    ("ragged_small", O.RED_SUM), ("ragged_small", O.RED_SEQ_MEAN), ("ragged_mid", O.RED_SUM),
])
def test_fused_matches_oracle_every_element(B, name, reduction):
    w = synth.workload(name)
    p = synth.hidden_problem(w)
    if name.startswith("tiny"):
        p["ids"] = _sample_ids_from_student(w, p)
    f = Hp.oracle_inputs(p)
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                      reduction=reduction, grad_scale=1.0, mode=w.mode)
    got = _run_fused(B, w, p, "cuda", reduction=reduction, grad_scale=1.0, dh_dtype=B.ADWIN_DT_F32)
    _check_fused(w, got, ref, reduction)


def test_fused_prefix_only_on_ragged_and_bf16_output_and_scale(B):
    import dataclasses
    w = dataclasses.replace(synth.workload("ragged_small"), mode=synth.MODE_PREFIX_ONLY)
    p = synth.hidden_problem(w)
    f = Hp.oracle_inputs(p)
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                      reduction=O.RED_SUM, grad_scale=-3.0, mode=w.mode)
    got = _run_fused(B, w, p, "cuda", reduction=O.RED_SUM, grad_scale=-3.0, dh_dtype=B.ADWIN_DT_BF16)
    _check_fused(w, got, ref, O.RED_SUM, dh_bf16=True)


def test_fused_is_deterministic_and_flags_bad_ids(B):
    w = synth.workload("ragged_small")
    p = synth.hidden_problem(w)
    a = _run_fused(B, w, p, "cuda", reduction=O.RED_SUM)
    b = _run_fused(B, w, p, "cuda", reduction=O.RED_SUM)
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    p["ids"] = p["ids"].clone()
    p["ids"][0] = w.V + 5
    c = _run_fused(B, w, p, "cuda", reduction=O.RED_SUM)
    assert int(c["status_dev"][0]) & B.ADWIN_DEV_BAD_ID
    assert c["c"][0] == 0.0 and np.array_equal(c["kl"], a["kl"])


def test_non_finite_rows_are_flagged_and_stay_local(B):
    """A row whose logits overflow (an infinite hidden state; logits thousands of nats apart, far
    beyond what exp(z - ref) holds) sets ADWIN_DEV_NONFINITE in status_dev; the other rows are
    what they are without it."""
    w = synth.workload("ragged_small")
    p = synth.hidden_problem(w)
    clean = _run_fused(B, w, p, "cuda", reduction=O.RED_SUM)
    assert int(clean["status_dev"][0]) == 0
    rows = O.plan(w.offsets, w.window)["rows"]
    for poison in (float("inf"), 3.0e4):
        q = dict(p)
        q["h_s"] = p["h_s"].clone()
        bad = int(rows[3])
        if poison == float("inf"):
            q["h_s"][bad, 7] = poison
        else:
            q["h_s"][bad] *= poison
        for scheme in (B.ADWIN_SCHEME_SINGLE, B.ADWIN_SCHEME_TWO_SWEEP):
            if scheme == B.ADWIN_SCHEME_TWO_SWEEP and poison != float("inf"):
                continue      # finite logits, however far apart, are in range for the running maximum
            got = _run_fused(B, w, q, "cuda", reduction=O.RED_SUM, scheme=scheme,
                             want=B.FusedCall.DEFAULT_OUTPUTS + (("dW_prefix", "t_entropy") if scheme == B.ADWIN_SCHEME_SINGLE else ()))
            assert int(got["status_dev"][0]) & B.ADWIN_DEV_NONFINITE, (poison, scheme)
            keep = np.ones(w.T, bool); keep[bad] = False
            ref_run = clean if scheme == B.ADWIN_SCHEME_SINGLE else _run_fused(B, w, p, "cuda", reduction=O.RED_SUM, scheme=scheme)
            assert np.array_equal(got["kl"][keep], ref_run["kl"][keep])
            assert np.array_equal(got["dh_prefix"][keep], ref_run["dh_prefix"][keep])
            # the row itself is excluded: zeros, and every reduced output stays finite and is that
            # of the batch without the row
            assert got["kl"][bad] == 0 and got["c"][bad] == 0 and not got["dh_prefix"][bad].any()
            assert not got["dh_full"][bad].any()
            for k, v in got.items():
                assert np.all(np.isfinite(v)), (k, poison, scheme)
            i_bad = int(np.searchsorted(w.offsets, bad, side="right") - 1)
            n_bad = min(int(w.window[i_bad]), int(w.offsets[i_bad + 1] - w.offsets[i_bad]))
            want_loss = ref_run["loss_prefix"].astype(np.float64).copy()
            want_loss[i_bad] -= float(ref_run["kl"][bad]) / n_bad
            assert np.allclose(got["loss_prefix"], want_loss, rtol=1e-5, atol=1e-6)
            others = np.arange(w.B) != i_bad
            assert np.allclose(got["rho_pooled"][others], ref_run["rho_pooled"][others], atol=1e-6)
    # a finite row far outside the single sweep's range is in range for the running maxima
    q = dict(p); q["h_s"] = p["h_s"].clone(); q["h_s"][int(rows[3])] *= 3.0e4
    got = _run_fused(B, w, q, "cuda", reduction=O.RED_SUM, scheme=B.ADWIN_SCHEME_TWO_SWEEP)
    assert int(got["status_dev"][0]) == 0
    fq = Hp.oracle_inputs(q)
    t = int(rows[3])
    kl_t = O.token_kl(fq["W_s"] @ fq["h_s"][t], fq["W_t"] @ fq["h_t"][t])
    assert abs(got["kl"][t] - kl_t) <= 2e-3 * kl_t          # logits of magnitude 1e4: fp32 rounding of z
    lo = synth.logits_problem(w)
    d = {k: v.cuda() for k, v in lo.items()}
    poisoned = d["z_s"].clone()
    poisoned[int(rows[3]), 5] = float("inf")
    for scheme in (B.ADWIN_LOGITS_RESIDENT, B.ADWIN_LOGITS_STREAMING):
        base = B.adwin_opd_from_logits(d["z_s"], d["z_t"], d["ids"], w.offsets, w.window, reduction=O.RED_SUM,
                                       scheme=scheme)
        torch.cuda.synchronize()
        base = {k: v.float().cpu().numpy() for k, v in base.items()}
        d_bad = dict(d, z_s=poisoned)
        out = B.adwin_opd_from_logits(d_bad["z_s"], d["z_t"], d["ids"], w.offsets, w.window, reduction=O.RED_SUM,
                                      scheme=scheme)
        torch.cuda.synchronize()
        assert int(out["status_dev"][0]) & B.ADWIN_DEV_NONFINITE
        o = {k: v.float().cpu().numpy() for k, v in out.items()}
        assert all(np.all(np.isfinite(v)) for v in o.values())
        assert o["kl"][int(rows[3])] == 0 and not o["dz"][int(rows[3])].any()
        keep = np.ones(w.T, bool); keep[int(rows[3])] = False
        assert np.array_equal(o["kl"][keep], base["kl"][keep]) and np.array_equal(o["dz"][keep], base["dz"][keep])


def test_teacher_equal_to_student_gives_zero(B):
    w = synth.workload("tiny_probe")
    p = synth.hidden_problem(w)
    d = {k: v.cuda() for k, v in p.items()}
    out = B.adwin_opd_fused(d["h_s"], d["h_s"], d["W_s"], d["W_s"], d["ids"], w.offsets, w.window,
                            mode=w.mode, reduction=B.ADWIN_RED_SUM)
    torch.cuda.synchronize()
    assert float(out["kl"].abs().max()) < 1e-5
    assert float(out["c"].abs().max()) < 1e-4
    assert float(out["dh_full"].abs().max()) < 1e-6


@pytest.mark.parametrize("name,reduction", [("tiny", O.RED_SUM), ("ragged_small", O.RED_SEQ_MEAN),
                                            ("ragged_mid", O.RED_TOKEN_MEAN)])
def test_logits_given_matches_oracle_every_element(B, name, reduction):
    w = synth.workload(name)
    p = synth.logits_problem(w)
    f = Hp.oracle_inputs(p)
    ref = O.supervise_from_logits(f["z_s"], f["z_t"], f["ids"], w.offsets, w.window,
                                  reduction=reduction, grad_scale=2.0)
    d = {k: v.cuda() for k, v in p.items()}
    out = B.adwin_opd_from_logits(d["z_s"], d["z_t"], d["ids"], w.offsets, w.window,
                                  reduction=reduction, grad_scale=2.0)
    torch.cuda.synchronize()
    got = {k: v.float().cpu().numpy() if v.dtype.is_floating_point else v.cpu().numpy()
           for k, v in out.items()}
    assert np.array_equal(got["n_out"], ref["n"]) and int(got["n_adm_out"][0]) == ref["n_adm"]
    assert int(got["status_dev"][0]) == 0
    Hp.assert_kl(got["kl"], ref["kl"])
    Hp.assert_cost(got["c"], ref["c"])
    Hp.assert_grad(got["dz"], ref["dz"], "dz", Hp.BF16_ULP)
    Hp.assert_close_rel(got["loss_prefix"], ref["loss_prefix"], Hp.LOSS_REL, "loss_prefix")
    Hp.assert_close_rel(got["batch"][:1], ref["batch"][:1], Hp.LOSS_REL, "L^p")
    assert np.all(got["batch"][1:] == 0)
    # shift invariance: adding a per-row constant to the teacher logits is what the
    # synthetic per-row shift does; KL must not see it (up to bf16 re-rounding of inputs)
    assert np.all(np.abs(got["dz"].astype(np.float64).sum(axis=1)) <=
                  1e-2 * np.abs(got["dz"]).sum(axis=1) + 1e-30)


@pytest.mark.parametrize("estimator", [O.EST_EXPECTED, O.EST_SAMPLED])
def test_logits_given_vocabulary_beyond_the_resident_capacity(B, estimator):
    """The row-resident kernel keeps 153,600 logits of a row pair on chip; a longer row reads
    the excess from memory in both sweeps.  V = 153,896: 37 vectors beyond the capacity, the
    last resident iteration full."""
    V = 153600 + 8 * 37
    w = synth.Workload("long_rows", V, 0, 0, synth._offsets([2, 0, 3]), np.array([2, 4, 2], np.int32))
    p = synth.logits_problem(w)
    f = Hp.oracle_inputs(p)
    ref = O.supervise_from_logits(f["z_s"], f["z_t"], f["ids"], w.offsets, w.window,
                                  reduction=O.RED_SUM, estimator=estimator)
    d = {k: v.cuda() for k, v in p.items()}
    out = B.adwin_opd_from_logits(d["z_s"], d["z_t"], d["ids"], w.offsets, w.window,
                                  reduction=O.RED_SUM, estimator=estimator)
    torch.cuda.synchronize()
    got = {k: v.float().cpu().numpy() if v.dtype.is_floating_point else v.cpu().numpy()
           for k, v in out.items()}
    assert int(got["status_dev"][0]) == 0 and int(got["n_adm_out"][0]) == 4
    Hp.assert_kl(got["kl"], ref["kl"])
    Hp.assert_cost(got["c"], ref["c"])
    Hp.assert_grad(got["dz"], ref["dz"], "dz", Hp.BF16_ULP)
    assert np.all(got["dz"][4] == 0)                      # the row outside its window
    Hp.assert_close_rel(got["loss_prefix"], ref["loss_prefix"], Hp.LOSS_REL, "loss_prefix")


@pytest.mark.parametrize("scheme", ["ADWIN_SCHEME_SINGLE", "ADWIN_SCHEME_TWO_SWEEP", "ADWIN_SCHEME_TWO_SWEEP_REG"])
def test_fallback_schemes_match_oracle(B, scheme):
    """The scheme field of the problem struct selects the single sweep, the two-sweep scheme
    (running maxima) or the latter with register-staged tiles; all meet the same bar."""
    scheme = getattr(B, scheme)
    w = synth.workload("ragged_small")
    p = synth.hidden_problem(w)
    f = Hp.oracle_inputs(p)
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                      reduction=O.RED_SUM, grad_scale=1.0, mode=w.mode)
    got = _run_fused(B, w, p, "cuda", reduction=O.RED_SUM, grad_scale=1.0, dh_dtype=B.ADWIN_DT_F32,
                     scheme=scheme)
    _check_fused(w, got, ref, O.RED_SUM)
    d = {k: v.cuda() for k, v in p.items()}
    call = B.FusedCall(d["h_s"], d["h_t"], d["W_s"], d["W_t"], d["ids"], w.offsets, w.window, mode=w.mode,
                       want=B.FusedCall.DEFAULT_OUTPUTS + ("t_entropy",), scheme=scheme)
    if scheme == B.ADWIN_SCHEME_SINGLE:
        assert call.run() == 0
    else:       # what rides on the single sweep is refused under the others
        assert call.run() == B.ADWIN_E_MODE
    # the workspace follows the scheme of the same struct
    single = B.FusedCall(d["h_s"], d["h_t"], d["W_s"], d["W_t"], d["ids"], w.offsets, w.window, mode=w.mode,
                         scheme=B.ADWIN_SCHEME_SINGLE, allocate=False)
    other = B.FusedCall(d["h_s"], d["h_t"], d["W_s"], d["W_t"], d["ids"], w.offsets, w.window, mode=w.mode,
                        scheme=scheme, allocate=False)
    assert (B.adwin_opd_workspace_bytes(single.p) == B.adwin_opd_workspace_bytes(other.p)) == (scheme == B.ADWIN_SCHEME_SINGLE)
    torch.cuda.synchronize()


@pytest.mark.parametrize("name,reduction", [
    ("tiny_probe", O.RED_SEQ_MEAN), ("ragged_small", O.RED_SUM), ("ragged_small", O.RED_TOKEN_MEAN),
    ("ragged_mid", O.RED_SEQ_MEAN),
])
def test_candidate_audit_matches_oracle(B, name, reduction):
    """rho(L) for a list of candidate windows from the one full-rollout pass (Sec. 4.2):
    per-rollout pooled / field cosines and the micro / macro aggregates."""
    import dataclasses
    w = dataclasses.replace(synth.workload(name), mode=synth.MODE_PREFIX_AND_FULL)
    p = synth.hidden_problem(w)
    f = Hp.oracle_inputs(p)
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                      reduction=reduction, grad_scale=1.0, mode=w.mode)
    lens = np.diff(w.offsets)
    cands = [1, 7, 64, 100, 128, 129, int(lens.max()), int(lens.max()) + 50]
    aud = O.audit_candidates(ref["g"], w.offsets, cands, reduction)
    got = _run_fused(B, w, p, "cuda", reduction=reduction, grad_scale=1.0, dh_dtype=B.ADWIN_DT_F32,
                     candidates=cands)
    _check_fused(w, got, ref, reduction)                 # the primary outputs are unchanged
    assert got["cand_rho_pooled"].shape == (len(cands), w.B)
    assert np.all(np.abs(got["cand_rho_pooled"] - aud["rho_pooled"]) <= Hp.RHO_ABS)
    assert np.all(np.abs(got["cand_rho_field"] - aud["rho_field"]) <= Hp.RHO_ABS)
    want = np.stack([aud["micro"], aud["micro_field"], aud["macro"], aud["macro_field"]], axis=1)
    assert np.all(np.abs(got["cand_batch"] - want) <= Hp.RHO_ABS), (got["cand_batch"], want)
    # a window that covers every rollout reproduces the full gradient: cosine 1
    nz = lens > 0
    assert np.all(np.abs(got["cand_rho_pooled"][-1][nz] - 1.0) <= 1e-5)
    # the scheduler picks the same window from either set of scores
    assert B.adwin_opd_next_window(got["cand_batch"][:, 0], cands) in \
        {O.next_window(aud["micro"], cands), O.next_window(aud["micro"] - 2 * Hp.RHO_ABS, cands),
         O.next_window(aud["micro"] + 2 * Hp.RHO_ABS, cands)}


def _teacher_reference(z_t, ids, rows, delta):
    """Oracle diagnostics of the given rows; the rank as a band [lo, hi] that absorbs logits
    within `delta` of the sampled token's (the two sides round the logits differently)."""
    ent, logp, lo, hi = {}, {}, {}, {}
    for t in rows:
        z, y = z_t[t], int(ids[t])
        ent[t], logp[t] = O.teacher_entropy(z), O.teacher_logp(z, y)
        exact = O.teacher_rank(z, y)
        near = np.abs(z - z[y]) <= delta
        near[y] = False
        lo[t] = exact - int(np.sum(near & (z > z[y])))
        hi[t] = exact + int(np.sum(near & (z <= z[y])))
    return ent, logp, lo, hi


@pytest.mark.parametrize("name", ["tiny_probe", "ragged_small", "ragged_mid"])
def test_teacher_diagnostics_fused(B, name):
    """Teacher entropy, rank of the sampled token and its teacher log-probability (Sec. 3.1)
    as by-products of the sweep."""
    w = synth.workload(name)
    p = synth.hidden_problem(w)
    f = Hp.oracle_inputs(p)
    want = ("kl", "c", "dh_prefix", "dh_full", "loss_prefix", "loss_full", "rho_pooled", "rho_field",
            "batch", "n_out", "n_adm_out", "status_dev", "t_logp", "t_entropy", "t_rank")
    got = _run_fused(B, w, p, "cuda", reduction=O.RED_SUM, want=want)
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                      reduction=O.RED_SUM, grad_scale=1.0, mode=w.mode)
    _check_fused(w, got, ref, O.RED_SUM)                 # the diagnostics mode changes nothing else
    z_t = f["h_t"] @ f["W_t"].T
    rows = list(ref["rows"])
    ent, logp, lo, hi = _teacher_reference(z_t, f["ids"], rows, 1e-4)
    for t in rows:
        assert abs(got["t_entropy"][t] - ent[t]) <= 1e-3, (t, got["t_entropy"][t], ent[t])
        assert abs(got["t_logp"][t] - logp[t]) <= 1e-3 * max(1.0, abs(logp[t]))
        assert lo[t] <= got["t_rank"][t] <= hi[t], (t, got["t_rank"][t], lo[t], hi[t])
    assert sum(hi[t] - lo[t] for t in rows) <= 3 * len(rows)  # the bands are narrow: a few near-ties per row
    other = np.setdiff1d(np.arange(w.T), ref["rows"])
    assert not got["t_entropy"][other].any() and not got["t_rank"][other].any()


def test_teacher_diagnostics_from_logits_exact_rank(B):
    w = synth.workload("ragged_small")
    p = synth.logits_problem(w)
    f = Hp.oracle_inputs(p)
    d = {k: v.cuda() for k, v in p.items()}
    want = ("kl", "c", "dz", "loss_prefix", "batch", "n_out", "n_adm_out", "status_dev",
            "t_logp", "t_entropy", "t_rank", "t_first_reject", "t_logp_mean")
    out = B.adwin_opd_from_logits(d["z_s"], d["z_t"], d["ids"], w.offsets, w.window,
                                  reduction=O.RED_SUM, want=want, topk=2000)
    torch.cuda.synchronize()
    got = {k: v.float().cpu().numpy() if v.dtype.is_floating_point else v.cpu().numpy()
           for k, v in out.items()}
    ref = O.supervise_from_logits(f["z_s"], f["z_t"], f["ids"], w.offsets, w.window, reduction=O.RED_SUM)
    Hp.assert_kl(got["kl"], ref["kl"])
    Hp.assert_grad(got["dz"], ref["dz"], "dz", Hp.BF16_ULP)
    rows = O.plan(w.offsets, w.window)["rows"]
    for t in rows:
        z, y = f["z_t"][t], int(f["ids"][t])
        assert got["t_rank"][t] == O.teacher_rank(z, y)                 # bf16 inputs: exact
        assert abs(got["t_entropy"][t] - O.teacher_entropy(z)) <= 1e-4
        assert abs(got["t_logp"][t] - O.teacher_logp(z, y)) <= 1e-4 * max(1.0, abs(O.teacher_logp(z, y)))
    other = np.setdiff1d(np.arange(w.T), rows)
    assert not got["t_entropy"][other].any() and not got["t_rank"][other].any()
    # rollout summaries over the admitted positions (ranks are exact here, so end to end);
    # ids are uniform, so ranks are too: k = 2000 of 8000 rejects most rollouts somewhere
    n = O.plan(w.offsets, w.window)["n"]
    fr = [O.first_rejection([O.teacher_rank(f["z_t"][t], int(f["ids"][t])) for t in range(w.offsets[i], w.offsets[i] + n[i])],
                            2000) for i in range(w.B)]
    assert np.array_equal(got["t_first_reject"], fr) and (np.array(fr) < n).any()
    logp = np.array([O.teacher_logp(f["z_t"][t], int(f["ids"][t])) for t in range(w.T)])
    assert np.allclose(got["t_logp_mean"], O.region_means(logp, w.offsets, n, n), rtol=1e-4, atol=1e-4)


@pytest.mark.parametrize("name,reduction", [("tiny", O.RED_SUM), ("tiny_probe", O.RED_SEQ_MEAN),
                                            ("ragged_small", O.RED_SUM), ("ragged_mid", O.RED_TOKEN_MEAN)])
def test_sampled_estimator_fused(B, name, reduction):
    """Eq. 4 on the sampled token, c_t (e_y - p_s), back to the hidden state; every other
    output as with the expected estimator."""
    w = synth.workload(name)
    p = synth.hidden_problem(w)
    if name.startswith("tiny"):
        p["ids"] = _sample_ids_from_student(w, p)
    f = Hp.oracle_inputs(p)
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                      reduction=reduction, grad_scale=1.0, mode=w.mode, estimator=O.EST_SAMPLED)
    got = _run_fused(B, w, p, "cuda", reduction=reduction, grad_scale=1.0, dh_dtype=B.ADWIN_DT_F32,
                     estimator=B.ADWIN_EST_SAMPLED)
    _check_fused(w, got, ref, reduction)
    exp = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                      reduction=reduction, grad_scale=1.0, mode=w.mode)
    assert np.abs(ref["dh_prefix"] - exp["dh_prefix"]).max() > 0.1 * np.abs(exp["dh_prefix"]).max()


@pytest.mark.parametrize("scheme", [0, 2])          # row-resident (default), streaming
def test_sampled_estimator_from_logits(B, scheme):
    w = synth.workload("ragged_small")
    p = synth.logits_problem(w)
    f = Hp.oracle_inputs(p)
    ref = O.supervise_from_logits(f["z_s"], f["z_t"], f["ids"], w.offsets, w.window,
                                  reduction=O.RED_SEQ_MEAN, grad_scale=-2.0, estimator=O.EST_SAMPLED)
    d = {k: v.cuda() for k, v in p.items()}
    out = B.adwin_opd_from_logits(d["z_s"], d["z_t"], d["ids"], w.offsets, w.window,
                                  reduction=O.RED_SEQ_MEAN, grad_scale=-2.0, estimator=B.ADWIN_EST_SAMPLED,
                                  scheme=scheme)
    torch.cuda.synchronize()
    got = {k: v.float().cpu().numpy() if v.dtype.is_floating_point else v.cpu().numpy()
           for k, v in out.items()}
    Hp.assert_kl(got["kl"], ref["kl"])
    Hp.assert_cost(got["c"], ref["c"])
    Hp.assert_grad(got["dz"], ref["dz"], "dz", Hp.BF16_ULP)
    rows = O.plan(w.offsets, w.window)["rows"]
    y = f["ids"][rows]
    # the one-hot entry carries the sign of c_t * scale, every other entry the opposite one
    assert np.all(np.sign(got["dz"][rows, y]) == np.sign(-2.0 * ref["c"][rows]))


def test_degenerate_batches(B):
    """Nothing admitted (all windows zero), and no rows at all: every output is defined and zero."""
    w = synth.workload("ragged_small")
    p = synth.hidden_problem(w)
    d = {k: v.cuda() for k, v in p.items()}
    zero_w = np.zeros(w.B, np.int32)
    out = B.adwin_opd_fused(d["h_s"], d["h_t"], d["W_s"], d["W_t"], d["ids"], w.offsets, zero_w,
                            mode=B.ADWIN_PREFIX_ONLY, reduction=B.ADWIN_RED_SEQ_MEAN,
                            want=("kl", "c", "dh_prefix", "loss_prefix", "loss_full", "rho_pooled", "rho_field",
                                  "batch", "n_out", "n_adm_out", "status_dev", "dW_prefix"))
    torch.cuda.synchronize()
    assert int(out["n_adm_out"][0]) == 0 and not out["n_out"].any() and int(out["status_dev"][0]) == 0
    for k in ("kl", "c", "dh_prefix", "loss_prefix", "loss_full", "rho_pooled", "rho_field", "batch", "dW_prefix"):
        assert not out[k].any(), k
    lo = synth.logits_problem(w)
    dl = {k: v.cuda() for k, v in lo.items()}
    out = B.adwin_opd_from_logits(dl["z_s"], dl["z_t"], dl["ids"], w.offsets, zero_w)
    torch.cuda.synchronize()
    assert not out["dz"].view(torch.int16).any() and not out["kl"].any() and not out["batch"].any()
    # no rows at all: three empty rollouts
    off0 = np.zeros(4, np.int64)
    e = {k: v[:0].contiguous() for k, v in d.items() if k in ("h_s", "h_t", "ids")}
    out = B.adwin_opd_fused(e["h_s"], e["h_t"], d["W_s"], d["W_t"], e["ids"], off0, np.array([5, 0, 9], np.int32),
                            mode=B.ADWIN_PREFIX_AND_FULL)
    torch.cuda.synchronize()
    assert int(out["n_adm_out"][0]) == 0 and not out["batch"].any() and not out["loss_full"].any()
    assert not out["rho_pooled"].any() and int(out["status_dev"][0]) == 0


WANT_HEAD = ("kl", "c", "dh_prefix", "dh_full", "loss_prefix", "loss_full", "rho_pooled", "rho_field",
             "batch", "n_out", "n_adm_out", "status_dev", "dW_prefix", "dW_full")


def _check_head_gradient(got, ref, probe, nrm):
    """nrm: Hp.summand_norms(..., head=True) of the same problem."""
    for k in ("dW_prefix", "dW_full") if probe else ("dW_prefix",):
        scale = np.abs(ref[k]).max()
        err = np.abs(got[k] - ref[k])
        tol = Hp.DW_SIGMAS * Hp.DW_SIGMA * nrm[k + "_l2"] + 1e-6 * scale
        assert (err <= tol).all(), (k, err.max(), scale, (err / tol).max())
        assert err.max() <= 2.0 ** -7 * scale
        # every dz row sums to zero over the vocabulary, so every column of dW does
        assert np.abs(got[k].astype(np.float64).sum(axis=0)).max() <= 1e-3 * np.abs(got[k]).sum(axis=0).max()
    if probe:      # the two objectives' alignment in the LM-head parameter block
        assert abs(got["batch"][6] - ref["rho_head"]) <= Hp.RHO_ABS, (got["batch"][6], ref["rho_head"])
        assert 0.0 < ref["rho_head"] < 1.0
    else:
        assert got["batch"][6] == 0


@pytest.mark.parametrize("name,reduction", [("tiny_probe", O.RED_SUM), ("ragged_small", O.RED_SEQ_MEAN),
                                            ("ragged_mid", O.RED_TOKEN_MEAN), ("tiny", O.RED_SUM)])
def test_head_weight_gradient(B, name, reduction):
    """dW_s of the prefix and of the full-rollout objective: the third contraction of the
    LM-head backward, sum_t w_t dz_t^T h_s[t]."""
    w = synth.workload(name)
    p = synth.hidden_problem(w)
    f = Hp.oracle_inputs(p)
    probe = w.mode == synth.MODE_PREFIX_AND_FULL
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                      reduction=reduction, grad_scale=-1.5, mode=w.mode, head_gradient=True)
    got = _run_fused(B, w, p, "cuda", reduction=reduction, grad_scale=-1.5, want=WANT_HEAD)
    _check_fused(w, got, ref, reduction)
    _check_head_gradient(got, ref, probe, Hp.summand_norms(f, w, ref["rows"], reduction, -1.5, head=True))


@pytest.mark.parametrize("name", ["tiny_probe", "ragged_small", "ragged_mid"])
def test_head_weight_gradient_sampled_estimator(B, name):
    """dW_s under Eq. 4's estimator: sum_t w_t c_t (e_{y_t} - p_s)^T h_s[t]."""
    w = synth.workload(name)
    p = synth.hidden_problem(w)
    f = Hp.oracle_inputs(p)
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                      reduction=O.RED_SEQ_MEAN, grad_scale=2.0, mode=w.mode, estimator=O.EST_SAMPLED,
                      head_gradient=True)
    got = _run_fused(B, w, p, "cuda", reduction=O.RED_SEQ_MEAN, grad_scale=2.0, want=WANT_HEAD,
                     estimator=B.ADWIN_EST_SAMPLED)
    _check_fused(w, got, ref, O.RED_SEQ_MEAN)
    _check_head_gradient(got, ref, True, Hp.summand_norms(f, w, ref["rows"], O.RED_SEQ_MEAN, 2.0, O.EST_SAMPLED, head=True))


def test_head_weight_gradient_accumulates_over_slabs(B, monkeypatch):
    """Rows split over several slabs: every slab adds its product to dW."""
    monkeypatch.setenv("ADWIN_SLAB_ROWS", "512")
    w = synth.workload("ragged_mid")
    p = synth.hidden_problem(w)
    d = {k: v.cuda() for k, v in p.items()}
    call = B.FusedCall(d["h_s"], d["h_t"], d["W_s"], d["W_t"], d["ids"], w.offsets, w.window, mode=w.mode,
                       reduction=O.RED_SUM, want=WANT_HEAD)
    assert B.adwin_opd_fused_launch_info(call.p)["slabs"] >= 4
    f = Hp.oracle_inputs(p)
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                      reduction=O.RED_SUM, mode=w.mode, head_gradient=True)
    nrm = Hp.summand_norms(f, w, ref["rows"], O.RED_SUM, head=True)
    first = None
    for _ in range(2):          # a second run over the same buffers overwrites, never adds to, the first
        assert call.run() == 0
        torch.cuda.synchronize()
        got = {k: v.float().cpu().numpy() if v.dtype.is_floating_point else v.cpu().numpy()
               for k, v in call.out.items()}
        _check_fused(w, got, ref, O.RED_SUM)
        _check_head_gradient(got, ref, True, nrm)
        if first is None:
            first = got
    for k in ("dW_prefix", "dW_full", "dh_full", "kl", "batch"):      # and reproduces it bit for bit
        assert np.array_equal(first[k], got[k]), k


@pytest.mark.parametrize("name", ["tiny", "tiny_probe", "ragged_small", "ragged_mid"])
def test_rollout_summaries(B, name):
    """First top-k rejection, prefix / suffix means of the teacher log-probability and the loss
    share inside every candidate window: the oracle's reductions applied to the call's own
    per-row outputs (which the tests above compare with the oracle row by row), and against
    the oracle end to end where no rank sits on a near-tie."""
    w = synth.workload(name)
    p = synth.hidden_problem(w)
    probe = w.mode == synth.MODE_PREFIX_AND_FULL
    cands = [1, 7, 64, 100, 300, 5000] if probe else None
    want = B.FusedCall.DEFAULT_OUTPUTS + ("t_logp", "t_entropy", "t_rank", "t_first_reject", "t_logp_mean")
    if probe:
        want += ("cand_loss_share",)
    K_TOP = 20                                     # the paper's evaluation-time top-k (Sec. 5.1)
    got = _run_fused(B, w, p, "cuda", reduction=O.RED_SUM, want=want, topk=K_TOP, candidates=cands)
    plan = O.plan(w.offsets, w.window)
    lens = np.diff(w.offsets)
    computed = lens if probe else plan["n"]
    ranks = [got["t_rank"][w.offsets[i]:w.offsets[i] + computed[i]] for i in range(w.B)]
    assert np.array_equal(got["t_first_reject"], [O.first_rejection(r, K_TOP) for r in ranks])
    assert (got["t_first_reject"] < computed).any()          # the case has rejections at all
    ref_mean = O.region_means(got["t_logp"].astype(np.float64), w.offsets, plan["n"], computed)
    assert np.allclose(got["t_logp_mean"], ref_mean, rtol=1e-6, atol=1e-6)
    if probe:
        ref_share = O.loss_share(got["kl"].astype(np.float64), w.offsets, computed, cands)
        assert np.allclose(got["cand_loss_share"], ref_share, rtol=1e-6, atol=1e-7)
        assert got["cand_loss_share"][-1] == pytest.approx(1.0, abs=1e-6)
        # end to end against the oracle: same tolerance class as the per-row quantities
        f = Hp.oracle_inputs(p)
        ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                          reduction=O.RED_SUM, mode=w.mode)
        assert np.allclose(got["cand_loss_share"], O.loss_share(ref["kl"], w.offsets, computed, cands),
                           rtol=Hp.KL_REL, atol=1e-6)
        z_t = f["h_t"] @ f["W_t"].T
        logp = np.array([O.teacher_logp(z_t[t], int(f["ids"][t])) for t in range(w.T)])
        assert np.allclose(got["t_logp_mean"], O.region_means(logp, w.offsets, plan["n"], computed),
                           rtol=1e-3, atol=1e-3)



@pytest.mark.parametrize("V,H_s,H_t,lens,win", [
    (8, 64, 64, [1], [1]),                        # the smallest legal problem: one token, 8 entries
    (40, 64, 128, [1, 3, 2], [1, 2, 5]),          # below one vocabulary tile, H below the image path
    (136, 128, 192, [5, 1], [3, 1]),              # one full vocabulary tile plus a tail of 8
    (264, 320, 128, [300], [257]),                # a window ending one row into the second token tile
])
def test_minimal_and_odd_shapes(B, V, H_s, H_t, lens, win):
    for mode in (synth.MODE_PREFIX_ONLY, synth.MODE_PREFIX_AND_FULL):
        w = synth.Workload(f"odd_{V}_{H_s}_{H_t}", V, H_s, H_t, synth._offsets(lens),
                           np.array(win, np.int32), mode)
        p = synth.hidden_problem(w)
        f = Hp.oracle_inputs(p)
        ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                          reduction=O.RED_SUM, mode=mode)
        got = _run_fused(B, w, p, "cuda", reduction=O.RED_SUM, dh_dtype=B.ADWIN_DT_F32)
        # A gradient element sums only V terms here, too few for the fraction-of-maximum bound
        # (stated for vocabularies where rounding averages out) to have its statistical margin:
        # every element is bounded by its own summands instead, as for the head-weight gradient.
        _check_fused(w, got, ref, O.RED_SUM, grad_l2=_grad_l2(f, w, ref, O.RED_SUM))
    lo = synth.logits_problem(w)
    fl = Hp.oracle_inputs(lo)
    d = {k: v.cuda() for k, v in lo.items()}
    out = B.adwin_opd_from_logits(d["z_s"], d["z_t"], d["ids"], w.offsets, w.window, reduction=O.RED_SUM)
    torch.cuda.synchronize()
    refl = O.supervise_from_logits(fl["z_s"], fl["z_t"], fl["ids"], w.offsets, w.window, reduction=O.RED_SUM)
    Hp.assert_kl(out["kl"].cpu().numpy(), refl["kl"])
    Hp.assert_grad(out["dz"].float().cpu().numpy(), refl["dz"], "dz", Hp.BF16_ULP)


def _random_shapes(n_cases, seed):
    g = np.random.default_rng(seed)
    cases = []
    for _ in range(n_cases):
        V = 8 * int(g.integers(1, 150, endpoint=True))
        H_s, H_t = (64 * int(g.integers(1, 7, endpoint=True)) for _ in range(2))
        nb = int(g.integers(1, 6, endpoint=True))
        lens = [int(g.integers(0, 400, endpoint=True)) if g.random() > 0.15 else 0 for _ in range(nb)]
        if sum(lens) == 0:
            lens[0] = 1
        win = [int(g.integers(0, l + 50, endpoint=True)) for l in lens]
        cases.append((V, H_s, H_t, lens, win, int(g.integers(0, 1, endpoint=True))))
    return cases


@pytest.mark.parametrize("V,H_s,H_t,lens,win,mode", _random_shapes(12, 20260528))
def test_random_small_shapes(B, V, H_s, H_t, lens, win, mode):
    """Seeded random shapes between the hand-picked ones: vocabularies of 8 .. 1200 entries, hidden
    sizes of 64 .. 448 (both logit kernels), empty rollouts, zero and over-long windows."""
    w = synth.Workload(f"rnd_{V}_{H_s}_{H_t}_{len(lens)}", V, H_s, H_t, synth._offsets(lens),
                       np.array(win, np.int32), mode)
    p = synth.hidden_problem(w)
    f = Hp.oracle_inputs(p)
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                      reduction=O.RED_SUM, mode=mode)
    got = _run_fused(B, w, p, "cuda", reduction=O.RED_SUM, dh_dtype=B.ADWIN_DT_F32)
    # vocabularies of at most 1,200 entries: gradient elements bounded by their own summands
    _check_fused(w, got, ref, O.RED_SUM, grad_l2=_grad_l2(f, w, ref, O.RED_SUM))


def test_every_output_is_optional(B):
    """NULL for an output means not wanted: each output alone equals the same output of a call
    that asks for everything."""
    w = synth.workload("ragged_small")
    p = synth.hidden_problem(w)
    d = {k: v.cuda() for k, v in p.items()}
    cands = [16, 200]
    everything = B.FusedCall.DEFAULT_OUTPUTS + ("t_logp", "t_entropy", "t_rank")

    def run(want):
        out = B.adwin_opd_fused(d["h_s"], d["h_t"], d["W_s"], d["W_t"], d["ids"], w.offsets, w.window,
                                mode=w.mode, want=want, candidates=cands)
        torch.cuda.synchronize()
        return {k: v.clone() for k, v in out.items()}
    full = run(everything)
    for k in everything:
        alone = run((k,))
        assert torch.equal(alone[k], full[k]), k
    lo = synth.logits_problem(w)
    dl = {k: v.cuda() for k, v in lo.items()}
    all_l = ("kl", "c", "dz", "loss_prefix", "batch", "n_out", "n_adm_out", "status_dev")
    full_l = B.adwin_opd_from_logits(dl["z_s"], dl["z_t"], dl["ids"], w.offsets, w.window, want=all_l)
    torch.cuda.synchronize()
    for k in all_l:
        alone = B.adwin_opd_from_logits(dl["z_s"], dl["z_t"], dl["ids"], w.offsets, w.window, want=(k,))
        torch.cuda.synchronize()
        a, b = alone[k], full_l[k]
        assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                           b.view(torch.int16) if b.dtype == torch.bfloat16 else b), k


def _peaked_workload():
    return synth.Workload("peaked", 8000, 256, 256, synth._offsets([150, 0, 300, 70]),
                          np.array([100, 5, 300, 20], np.int32), synth.MODE_PREFIX_AND_FULL)


@pytest.mark.parametrize("on_policy", [True, False])
@pytest.mark.parametrize("estimator", [O.EST_EXPECTED, O.EST_SAMPLED])
def test_peaked_distributions(B, estimator, on_policy):
    """Logits with a spread of 4 nats (half the mass on one entry, row maximum 14 nats on average
    and up to 25 above the largest of the first 128 entries) and a teacher that is a perturbed
    copy of the student: the regime of trained models, where the fixed references of the
    single sweep sit far below the row maximum and a gradient row is carried by a handful of
    vocabulary entries.  The gradients are held to the same bar as everywhere else (2e-3 of the
    largest element): the entries with p_s >= 1/32 are contracted in fp32."""
    w = _peaked_workload()
    p = synth.peaked_problem(w)
    if on_policy:                       # y_t ~ p_s, as in the method; else uniform over the vocabulary
        p["ids"] = _sample_ids_from_student(w, p)
    f = Hp.oracle_inputs(p)
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                      reduction=O.RED_SUM, mode=w.mode, estimator=estimator, head_gradient=True)
    assert 0.5 < ref["kl"].mean() < 3.0
    want = B.FusedCall.DEFAULT_OUTPUTS + ("t_logp", "t_entropy", "t_rank", "dW_prefix", "dW_full")
    got = _run_fused(B, w, p, "cuda", reduction=O.RED_SUM, dh_dtype=B.ADWIN_DT_F32, estimator=estimator,
                     want=want)
    z_t = f["h_t"] @ f["W_t"].T
    lse_t = np.array([np.log(np.exp(z - z.max()).sum()) + z.max() for z in z_t])
    _check_fused(w, got, ref, O.RED_SUM, logit_scale=np.abs(lse_t), abs_cap=False)
    _check_head_gradient(got, ref, True, Hp.summand_norms(f, w, ref["rows"], O.RED_SUM, 1.0, estimator, head=True))
    ent, logp, lo, hi = _teacher_reference(z_t, f["ids"], list(ref["rows"]), 1e-3)
    for t in ref["rows"]:
        assert abs(got["t_entropy"][t] - ent[t]) <= 2e-3, (t, got["t_entropy"][t], ent[t])
        assert abs(got["t_logp"][t] - logp[t]) <= 1e-3 * max(1.0, abs(logp[t]))
        assert lo[t] <= got["t_rank"][t] <= hi[t]


def test_peaked_distributions_other_paths(B):
    """The same peaked pair through the logits-given kernels (both) and through the two-sweep
    schemes of the fused path."""
    w = _peaked_workload()
    p = synth.peaked_problem(w)
    p["ids"] = _sample_ids_from_student(w, p)
    f = Hp.oracle_inputs(p)
    z_s = torch.from_numpy(f["h_s"] @ f["W_s"].T).to(torch.bfloat16)
    z_t = torch.from_numpy(f["h_t"] @ f["W_t"].T).to(torch.bfloat16)
    fz_s, fz_t = synth.to_f64(z_s), synth.to_f64(z_t)
    refl = O.supervise_from_logits(fz_s, fz_t, f["ids"], w.offsets, w.window, reduction=O.RED_SUM)
    lse = np.array([np.log(np.exp(z - z.max()).sum()) + z.max() for z in fz_t])
    for scheme in (B.ADWIN_LOGITS_RESIDENT, B.ADWIN_LOGITS_STREAMING):
        out = B.adwin_opd_from_logits(z_s.cuda(), z_t.cuda(), p["ids"].cuda(), w.offsets, w.window,
                                      reduction=O.RED_SUM, scheme=scheme)
        torch.cuda.synchronize()
        Hp.assert_kl(out["kl"].cpu().numpy(), refl["kl"], logit_scale=np.abs(lse))
        Hp.assert_cost(out["c"].cpu().numpy(), refl["c"])
        Hp.assert_grad(out["dz"].float().cpu().numpy(), refl["dz"], "dz", Hp.BF16_ULP, abs_cap=False)
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                      reduction=O.RED_SUM, mode=w.mode)
    lse_t = np.array([np.log(np.exp(z - z.max()).sum()) + z.max() for z in f["h_t"] @ f["W_t"].T])
    for scheme in (B.ADWIN_SCHEME_TWO_SWEEP, B.ADWIN_SCHEME_TWO_SWEEP_REG):
        got = _run_fused(B, w, p, "cuda", reduction=O.RED_SUM, dh_dtype=B.ADWIN_DT_F32, scheme=scheme)
        _check_fused(w, got, ref, O.RED_SUM, logit_scale=np.abs(lse_t), abs_cap=False)


@pytest.mark.parametrize("name", ["ragged_small", "ragged_mid", "tiny"])
def test_statistics_only_call(B, name):
    """No requested output depends on the gradients: the call runs the sweep without storing or
    contracting gradient factors, needs a smaller workspace, and returns the same values."""
    w = synth.workload(name)
    p = synth.hidden_problem(w)
    d = {k: v.cuda() for k, v in p.items()}
    probe = w.mode == synth.MODE_PREFIX_AND_FULL
    fwd = ("kl", "c", "loss_prefix", "loss_full", "n_out", "n_adm_out", "status_dev",
           "t_logp", "t_entropy", "t_rank", "t_first_reject", "t_logp_mean")
    if probe:
        fwd += ("cand_loss_share",)
    else:
        fwd += ("batch",)
    cands = [5, 64, 300] if probe else None
    full = B.FusedCall(d["h_s"], d["h_t"], d["W_s"], d["W_t"], d["ids"], w.offsets, w.window, mode=w.mode,
                       want=fwd + ("dh_prefix",), topk=50, candidates=cands)
    only = B.FusedCall(d["h_s"], d["h_t"], d["W_s"], d["W_t"], d["ids"], w.offsets, w.window, mode=w.mode,
                       want=fwd, topk=50, candidates=cands, cand_outputs=False)
    assert only.workspace_bytes < full.workspace_bytes
    assert full.run() == 0 and only.run() == 0
    torch.cuda.synchronize()
    for k in fwd:
        assert torch.equal(only.out[k], full.out[k]), k
    f = Hp.oracle_inputs(p)
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window, mode=w.mode)
    Hp.assert_kl(only.out["kl"].cpu().numpy(), ref["kl"])
    Hp.assert_close_rel(only.out["loss_prefix"].cpu().numpy(), ref["loss_prefix"], Hp.LOSS_REL, "loss_prefix")


def test_many_short_rollouts(B):
    """1,500 rollouts of 0..30 tokens (many empty, many with window 0 or beyond the end): the
    per-rollout kernels, the chunked pooled sums and the candidate audit at a large B."""
    g = np.random.default_rng(20260528)
    nb = 1500
    lens = g.integers(0, 30, size=nb, endpoint=True)
    win = g.integers(0, 40, size=nb, endpoint=True).astype(np.int32)
    w = synth.Workload("many_short", 264, 128, 128, synth._offsets(lens), win, synth.MODE_PREFIX_AND_FULL)
    p = synth.hidden_problem(w)
    f = Hp.oracle_inputs(p)
    cands = [1, 3, 8, 20, 64]
    for reduction in (O.RED_SEQ_MEAN, O.RED_TOKEN_MEAN):
        ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                          reduction=reduction, mode=w.mode)
        got = _run_fused(B, w, p, "cuda", reduction=reduction, dh_dtype=B.ADWIN_DT_F32, candidates=cands,
                         want=B.FusedCall.DEFAULT_OUTPUTS + ("t_rank", "t_logp", "t_first_reject", "t_logp_mean",
                                                            "cand_loss_share"), topk=100)
        # gradient elements: V = 264 is a tiny vocabulary (see test_minimal_and_odd_shapes)
        _check_fused(w, got, ref, reduction, grad_l2=_grad_l2(f, w, ref, reduction))
        aud = O.audit_candidates(ref["g"], w.offsets, cands, reduction)
        assert np.all(np.abs(got["cand_rho_pooled"] - aud["rho_pooled"]) <= Hp.RHO_ABS)
        assert np.all(np.abs(got["cand_rho_field"] - aud["rho_field"]) <= Hp.RHO_ABS)
        comp = lens
        ranks = [got["t_rank"][w.offsets[i]:w.offsets[i + 1]] for i in range(nb)]
        assert np.array_equal(got["t_first_reject"], [O.first_rejection(r, 100) for r in ranks])
        assert np.allclose(got["cand_loss_share"], O.loss_share(got["kl"].astype(np.float64), w.offsets, comp, cands),
                           rtol=1e-6, atol=1e-7)


def test_one_long_rollout(B):
    """A single rollout of 70,000 tokens (several slabs at the forced slab size, hundreds of
    reduction chunks): windows and candidates far inside, at and beyond its end."""
    w = synth.Workload("one_long", 264, 128, 128, synth._offsets([70000]), np.array([33333], np.int32),
                       synth.MODE_PREFIX_AND_FULL)
    p = synth.hidden_problem(w)
    f = Hp.oracle_inputs(p)
    cands = [1, 1000, 33333, 65536, 100000]
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], f["ids"], w.offsets, w.window,
                      reduction=O.RED_SEQ_MEAN, mode=w.mode, block=256)
    got = _run_fused(B, w, p, "cuda", reduction=O.RED_SEQ_MEAN, dh_dtype=B.ADWIN_DT_F32, candidates=cands)
    _check_fused(w, got, ref, O.RED_SEQ_MEAN, grad_l2=_grad_l2(f, w, ref, O.RED_SEQ_MEAN))
    aud = O.audit_candidates(ref["g"], w.offsets, cands, O.RED_SEQ_MEAN)
    assert np.all(np.abs(got["cand_rho_pooled"] - aud["rho_pooled"]) <= Hp.RHO_ABS)
    assert np.all(np.abs(got["cand_rho_field"] - aud["rho_field"]) <= Hp.RHO_ABS)
    assert abs(got["cand_rho_pooled"][2, 0] - got["rho_pooled"][0]) <= 1e-6       # the call's own window
    assert got["cand_rho_field"][3, 0] < 1.0 and got["cand_rho_field"][4, 0] == pytest.approx(1.0, abs=1e-6)
