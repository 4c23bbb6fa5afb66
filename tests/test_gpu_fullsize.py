"""GPU parity at the benchmark's full sizes (V = 151,936), in the launch configuration
bench.py times.  The oracle cannot sweep these in full, so per-token outputs are compared on
a seeded sample of 512 rows (window edges always included), integer outputs in full, the
window losses and alignment scores of whole short rollouts end to end against the oracle run
on those rollouts' rows, and those of all the other rollouts by applying the oracle's
reduction to the GPU's own per-row values ("reduction parity")."""
import numpy as np
import pytest
import torch

from oracle import adwin_oracle as O
from paper_2605_28396_amd import synth
from tests import helpers as Hp

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

K_ROWS = 512


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available()
    from paper_2605_28396_amd import binding
    return binding


def _free():
    import gc
    gc.collect()
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name,estimator", [("strong_to_weak", 0), ("same_family", 0),
                                            ("probe_alignment", 0), ("strong_to_weak", 1)])
def test_fused_full_size_sampled_rows_and_reductions(B, name, estimator):
    print(f"[case] fused full size {name} estimator {estimator}", flush=True)
    w = synth.workload(name)
    dev = torch.device("cuda:0")
    p = synth.hidden_problem(w, dev)
    probe = w.mode == synth.MODE_PREFIX_AND_FULL
    cands = list(O.CANDIDATE_WINDOWS) if probe else None
    want = B.FusedCall.DEFAULT_OUTPUTS
    if probe:       # the audit step also takes the teacher-side diagnostics and their summaries
        want += ("t_logp", "t_entropy", "t_rank", "t_first_reject", "t_logp_mean", "cand_loss_share")
    head = estimator == 0 and name in ("strong_to_weak", "probe_alignment")
    if head:        # the head-weight gradient(s) over all slabs, checked by identities below
        want += ("dW_prefix", "dW_full") if probe else ("dW_prefix",)
    call = B.FusedCall(p["h_s"], p["h_t"], p["W_s"], p["W_t"], p["ids"], w.offsets, w.window,
                       mode=w.mode, reduction=B.ADWIN_RED_SUM, dh_dtype=B.ADWIN_DT_F32,
                       candidates=cands, estimator=estimator, want=want, topk=20)
    st = call.run()
    assert st == 0, B.adwin_opd_strerror(st)
    torch.cuda.synchronize()
    out = call.out
    # integers, in full
    plan = O.plan(w.offsets, w.window)
    assert np.array_equal(out["n_out"].cpu().numpy(), plan["n"])
    assert int(out["n_adm_out"][0]) == plan["n_adm"]
    assert int(out["status_dev"][0]) == 0
    # sampled rows against the oracle
    rows = synth.sample_rows(w, K_ROWS)
    idx = torch.from_numpy(rows).to(dev)
    Ws, Wt = synth.to_f64(p["W_s"]), synth.to_f64(p["W_t"])
    kl, c, g = O.rows_terms(synth.to_f64(p["h_s"][idx]), synth.to_f64(p["h_t"][idx]), Ws, Wt,
                            p["ids"][idx].cpu().numpy(), estimator=estimator, block=64)
    print(f"[case] {len(rows)} sampled rows through the oracle", flush=True)
    Hp.assert_kl(out["kl"][idx].cpu().numpy(), kl)
    Hp.assert_cost(out["c"][idx].cpu().numpy(), c)
    adm = np.zeros(w.T, bool); adm[plan["rows"]] = True
    key = "dh_full" if probe else "dh_prefix"
    Hp.assert_grad(out[key][idx].cpu().numpy(), g, key)
    if probe:
        g_p = g * adm[rows][:, None]
        Hp.assert_grad(out["dh_prefix"][idx].cpu().numpy(), g_p, "dh_prefix")
    # Whole rollouts end to end (Sec. 4.1 window loss; Sec. 4.2 cosines): the oracle on every
    # computed row of the rollouts with the fewest computed rows -- two in the prefix-only
    # configurations, one in the full-rollout configuration -- as a batch of their own
    # (per-rollout losses and cosines do not depend on the rest of the batch under RED_SUM).
    lens = np.diff(w.offsets)
    if estimator == 0:
        computed = lens if probe else plan["n"]
        order = [int(i) for i in np.argsort(computed, kind="stable") if computed[i] > 0]
        for i in order[:1 if probe else 2]:
            o, m = int(w.offsets[i]), int(computed[i])
            sl = slice(o, o + m)
            one = O.supervise(synth.to_f64(p["h_s"][sl]), synth.to_f64(p["h_t"][sl]), Ws, Wt,
                              p["ids"][sl].cpu().numpy(), np.array([0, m]), np.array([int(w.window[i])]),
                              reduction=O.RED_SUM, mode=w.mode, block=64)
            print(f"[case] rollout {i}: {m} rows through the oracle", flush=True)
            Hp.assert_close_rel(out["loss_prefix"][i:i + 1].cpu().numpy(), one["loss_prefix"], Hp.LOSS_REL,
                                f"loss_prefix[{i}]")
            Hp.assert_kl(out["kl"][sl].cpu().numpy(), one["kl"])
            Hp.assert_grad(out["dh_prefix"][sl].cpu().numpy(), one["dh_prefix"], f"dh_prefix of rollout {i}")
            if probe:
                Hp.assert_close_rel(out["loss_full"][i:i + 1].cpu().numpy(), one["loss_full"], Hp.LOSS_REL,
                                    f"loss_full[{i}]")
                assert abs(float(out["rho_pooled"][i]) - one["rho_pooled"][0]) <= Hp.RHO_ABS, (i, one["rho_pooled"])
                assert abs(float(out["rho_field"][i]) - one["rho_field"][0]) <= Hp.RHO_ABS, (i, one["rho_field"])
                aud = O.audit_candidates(one["g"], np.array([0, m]), cands, O.RED_SUM)
                assert np.all(np.abs(out["cand_rho_pooled"][:, i].cpu().numpy() - aud["rho_pooled"][:, 0]) <= Hp.RHO_ABS)
                assert np.all(np.abs(out["cand_rho_field"][:, i].cpu().numpy() - aud["rho_field"][:, 0]) <= Hp.RHO_ABS)
            del one
    del Ws, Wt
    # rows outside the windows are exactly zero (sampled: first non-admitted row of each rollout)
    outside = [int(w.offsets[i] + plan["n"][i]) for i in range(w.B) if plan["n"][i] < lens[i]][:32]
    if outside:
        oi = torch.tensor(outside, device=dev)
        assert not bool(out["dh_prefix"][oi].any())
        if not probe:
            assert not bool(out["kl"][oi].any()) and not bool(out["c"][oi].any())
    if head:
        # dW and dh contract the same dz: <dW, W_s> = sum_t <dh[t], h_s[t]> (both sides are
        # sum_t w_t dz_t W_s h_s[t]); dh is compared with the oracle above, so this ties every
        # slab and tile of the third contraction to it.  Every dz row sums to zero, so every
        # column of dW does.
        for kW, kh in (("dW_prefix", "dh_prefix"), ("dW_full", "dh_full")) if probe else (("dW_prefix", "dh_prefix"),):
            dW = out[kW]
            lhs = float((dW.double() * p["W_s"].double()).sum())
            prod = out[kh].double() * p["h_s"].double()
            rhs, scale = float(prod.sum()), float(prod.abs().sum())
            del prod
            assert abs(lhs - rhs) <= 1e-3 * abs(rhs) + 1e-6 * scale, (kW, lhs, rhs, scale)
            assert abs(rhs) > 1e-3 * scale          # the identity is not a comparison of two noises
            col = dW.double().sum(dim=0).abs().max()
            assert float(col) <= 1e-3 * float(dW.double().abs().sum(dim=0).max()), kW
            del dW
        if probe:   # the two objectives' alignment in the head block, from the call's own gradients
            a, b = out["dW_prefix"].double(), out["dW_full"].double()
            cos = float((a * b).sum() / (a.norm() * b.norm()))
            del a, b
            assert abs(float(out["batch"][6]) - cos) <= 1e-5 and 0.0 < cos < 1.0
    # reduction parity: the oracle's window reduction applied to the GPU's per-row values
    kl_gpu = out["kl"].double().cpu().numpy()
    if probe:
        g_gpu = out["dh_full"].double().cpu().numpy()
    else:
        g_gpu = out["dh_prefix"].double().cpu().numpy()
    ref = O.window_outputs(kl_gpu, g_gpu, w.offsets, w.window, O.RED_SUM, 1.0, w.mode)
    Hp.assert_close_rel(out["loss_prefix"].cpu().numpy(), ref["loss_prefix"], 1e-5, "loss_prefix")
    Hp.assert_close_rel(out["batch"][:2].cpu().numpy(), ref["batch"][:2], 1e-5, "batch loss")
    if probe:
        Hp.assert_close_rel(out["loss_full"].cpu().numpy(), ref["loss_full"], 1e-5, "loss_full")
        for k in ("rho_pooled", "rho_field"):
            assert np.all(np.abs(out[k].cpu().numpy() - ref[k]) <= 1e-4), k
        assert np.all(np.abs(out["batch"][2:6].cpu().numpy() - ref["batch"][2:6]) <= 1e-4)
        rp = out["rho_pooled"].cpu().numpy()
        assert np.all(rp <= 1 + 1e-6) and np.all(rp >= -1 - 1e-6)
        # candidate audit (the paper's candidate list): per-rollout scores of the two shortest
        # rollouts against the oracle's audit of those rollouts' gradients; aggregates by
        # their defining properties
        crp = out["cand_rho_pooled"].cpu().numpy()
        crf = out["cand_rho_field"].cpu().numpy()
        cb = out["cand_batch"].cpu().numpy()
        for i in np.argsort(lens)[:2]:
            o, n = int(w.offsets[i]), int(lens[i])
            aud = O.audit_candidates(g_gpu[o:o + n], np.array([0, n]), cands, O.RED_SUM)
            assert np.all(np.abs(crp[:, i] - aud["rho_pooled"][:, 0]) <= 1e-4), (i, crp[:, i])
            assert np.all(np.abs(crf[:, i] - aud["rho_field"][:, 0]) <= 1e-4), (i, crf[:, i])
        assert np.all(np.abs(cb[:, 2] - crp.mean(axis=1)) <= 1e-5)      # macro = mean over rollouts
        assert np.all(np.abs(cb[:, 3] - crf.mean(axis=1)) <= 1e-5)
        assert np.all(np.diff(crf, axis=0) >= -1e-6)                    # field cosine grows with L
        # diagnostics on the sampled rows, their summaries by the oracle's reductions of the
        # call's own per-row values
        z_rows = synth.to_f64(p["h_t"][idx]) @ synth.to_f64(p["W_t"]).T
        ids_rows = p["ids"][idx].cpu().numpy()
        t_ent, t_lp, t_rk = (out[k][idx].cpu().numpy() for k in ("t_entropy", "t_logp", "t_rank"))
        for q in range(0, len(rows), 8):
            assert abs(t_ent[q] - O.teacher_entropy(z_rows[q])) <= 1e-3
            lp = O.teacher_logp(z_rows[q], int(ids_rows[q]))
            assert abs(t_lp[q] - lp) <= 1e-3 * max(1.0, abs(lp))
            above = int(np.sum(z_rows[q] > z_rows[q][ids_rows[q]] + 1e-3))
            near = int(np.sum(np.abs(z_rows[q] - z_rows[q][ids_rows[q]]) <= 1e-3))
            assert above + 1 <= t_rk[q] <= above + near
        del z_rows
        rk = out["t_rank"].cpu().numpy()
        fr = [O.first_rejection(rk[w.offsets[i]:w.offsets[i + 1]], 20) for i in range(w.B)]
        assert np.array_equal(out["t_first_reject"].cpu().numpy(), fr)
        ref_mean = O.region_means(out["t_logp"].double().cpu().numpy(), w.offsets, plan["n"], lens)
        assert np.allclose(out["t_logp_mean"].cpu().numpy(), ref_mean, rtol=1e-5, atol=1e-5)
        ref_share = O.loss_share(kl_gpu, w.offsets, lens, cands)
        assert np.allclose(out["cand_loss_share"].cpu().numpy(), ref_share, rtol=1e-5, atol=1e-6)
        k2048 = cands.index(2048)                                       # the call's own window
        assert np.all(np.abs(crp[k2048] - rp) <= 1e-5)
        assert np.all(np.abs(cb[k2048] - out["batch"][2:6].cpu().numpy()) <= 1e-5)
    del call, out, p
    _free()


def test_fused_full_size_peaked_rows(B):
    """The benchmark shape with a peaked same-family pair instead of random-initialisation
    tensors (half the mass of a row on one entry, row maximum far above the first vocabulary
    entries, ids uniform, i.e. the references get no help from the sampled token): sampled
    rows against the oracle at the standard bar."""
    print("[case] fused full size, peaked rows", flush=True)
    w = synth.workload("strong_to_weak")
    dev = torch.device("cuda:0")
    p = synth.peaked_problem(w, dev)
    call = B.FusedCall(p["h_s"], p["h_t"], p["W_s"], p["W_t"], p["ids"], w.offsets, w.window,
                       mode=w.mode, reduction=B.ADWIN_RED_SUM, dh_dtype=B.ADWIN_DT_F32)
    assert call.run() == 0
    torch.cuda.synchronize()
    out = call.out
    assert int(out["status_dev"][0]) == 0
    rows = synth.sample_rows(w, 256)
    idx = torch.from_numpy(rows).to(dev)
    Ws, Wt = synth.to_f64(p["W_s"]), synth.to_f64(p["W_t"])
    hs, ht = synth.to_f64(p["h_s"][idx]), synth.to_f64(p["h_t"][idx])
    kl, c, g = O.rows_terms(hs, ht, Ws, Wt, p["ids"][idx].cpu().numpy(), block=64)
    assert 0.3 < kl.mean() < 5.0
    lse_t = np.array([np.log(np.exp(z - z.max()).sum()) + z.max() for z in ht[::16] @ Wt.T])
    del Ws, Wt
    Hp.assert_kl(out["kl"][idx].cpu().numpy(), kl, logit_scale=np.abs(lse_t).max())
    Hp.assert_cost(out["c"][idx].cpu().numpy(), c)
    # the same bar as for flat rows, relative to the largest element (gradients of order 1 here)
    Hp.assert_grad(out["dh_prefix"][idx].double().cpu().numpy(), g, "dh_prefix", abs_cap=False)
    del call, out, p
    _free()


def test_head_weight_gradient_full_vocabulary(B):
    """dW_s at the benchmark's vocabulary size (all 594 vocabulary tiles; 4 hidden tiles) over a
    batch and hidden sizes small enough for the oracle: every row feeds every element, so rows
    cannot be sampled; the batch is what is reduced."""
    print("[case] head-weight gradient, full vocabulary", flush=True)
    full = synth.workload("strong_to_weak")
    lens = [40, 0, 70, 21]
    w = synth.Workload("head_full_vocab", full.V, 1024, 1024, synth._offsets(lens),
                       np.array([30, 7, 100, 0], np.int32))
    dev = torch.device("cuda:0")
    p = synth.hidden_problem(w, dev)
    want = ("kl", "c", "dh_prefix", "loss_prefix", "loss_full", "rho_pooled", "rho_field", "batch",
            "n_out", "n_adm_out", "status_dev", "dW_prefix")
    call = B.FusedCall(p["h_s"], p["h_t"], p["W_s"], p["W_t"], p["ids"], w.offsets, w.window,
                       mode=w.mode, reduction=B.ADWIN_RED_SEQ_MEAN, grad_scale=3.0, dh_dtype=B.ADWIN_DT_F32,
                       want=want)
    assert call.run() == 0
    torch.cuda.synchronize()
    f = {k: synth.to_f64(p[k]) for k in ("h_s", "h_t", "W_s", "W_t")}
    ref = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], p["ids"].cpu().numpy(), w.offsets, w.window,
                      reduction=O.RED_SEQ_MEAN, grad_scale=3.0, mode=w.mode, head_gradient=True, block=128)
    print("[case] oracle done", flush=True)
    got = call.out["dW_prefix"].double().cpu().numpy()
    scale = np.abs(ref["dW_prefix"]).max()
    err = np.abs(got - ref["dW_prefix"])
    fi = dict(f, ids=p["ids"].cpu().numpy())
    l2 = Hp.summand_norms(fi, w, ref["rows"], O.RED_SEQ_MEAN, 3.0, head=True, block=32)["dW_prefix_l2"]
    tol = Hp.DW_SIGMAS * Hp.DW_SIGMA * l2 + 1e-6 * scale
    assert (err <= tol).all(), (err.max(), scale, (err / tol).max())
    Hp.assert_grad(call.out["dh_prefix"].cpu().numpy(), ref["dh_prefix"], "dh_prefix")
    del call, p, f, ref
    _free()



def test_logits_given_full_size_sampled_rows(B):
    print("[case] logits-given full size", flush=True)
    w = synth.workload("logits_given")
    dev = torch.device("cuda:0")
    p = synth.logits_problem(w, dev)
    call = B.LogitsCall(p["z_s"], p["z_t"], p["ids"], w.offsets, w.window, reduction=B.ADWIN_RED_SUM)
    st = call.run()
    assert st == 0, B.adwin_opd_strerror(st)
    torch.cuda.synchronize()
    out = call.out
    plan = O.plan(w.offsets, w.window)
    assert np.array_equal(out["n_out"].cpu().numpy(), plan["n"])
    assert int(out["n_adm_out"][0]) == plan["n_adm"] and int(out["status_dev"][0]) == 0
    rows = synth.sample_rows(w, 96)
    idx = torch.from_numpy(rows).to(dev)
    zs, zt = synth.to_f64(p["z_s"][idx]), synth.to_f64(p["z_t"][idx])
    ids = p["ids"][idx].cpu().numpy()
    kl = np.array([O.token_kl(zs[r], zt[r]) for r in range(len(rows))])
    c = np.array([O.token_cost(zs[r], zt[r], int(ids[r])) for r in range(len(rows))])
    dz = np.stack([O.token_dz(zs[r], zt[r]) for r in range(len(rows))])
    Hp.assert_kl(out["kl"][idx].cpu().numpy(), kl)
    Hp.assert_cost(out["c"][idx].cpu().numpy(), c)
    Hp.assert_grad(out["dz"][idx].float().cpu().numpy(), dz, "dz", Hp.BF16_ULP)
    # rows outside the windows: zero gradient, zero KL (all of them)
    adm = torch.zeros(w.T, dtype=torch.bool, device=dev)
    adm[torch.from_numpy(plan["rows"]).to(dev)] = True
    assert not bool(out["kl"][~adm].any())
    nz = out["dz"].view(torch.int16).ne(0).any(dim=1)
    assert bool((nz == adm).all())
    # window losses from the GPU's own per-token KL
    kl_gpu = out["kl"].double().cpu().numpy()
    for i in range(w.B):
        o, ni = int(w.offsets[i]), int(plan["n"][i])
        want = kl_gpu[o:o + ni].mean() if ni else 0.0
        assert abs(float(out["loss_prefix"][i]) - want) <= 1e-5 * abs(want) + 1e-7
    assert abs(float(out["batch"][0]) - kl_gpu.sum()) <= 1e-5 * kl_gpu.sum()
    del call, out, p
    _free()
