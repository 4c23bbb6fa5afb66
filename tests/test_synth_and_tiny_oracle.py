"""Input recipe checks and the oracle run end-to-end on the Tiny configuration."""
import numpy as np
import torch

from oracle import adwin_oracle as O
from paper_2605_28396_amd import synth


def test_workload_shapes_match_the_stated_configs():
    w = synth.workload("tiny")
    assert (w.B, w.T, w.V, w.H_s, w.H_t) == (2, 224, 4096, 256, 384)
    assert w.window.tolist() == [64, 128]
    w = synth.workload("logits_given")
    lens = np.diff(w.offsets)
    assert w.B == 32 and w.T == 32768 and lens.min() >= 256 and lens.max() <= 2048
    assert np.all(w.window >= 64) and np.all(w.window <= lens)
    w = synth.workload("strong_to_weak")
    lens = np.diff(w.offsets)
    assert w.B == 64 and lens.min() >= 1024 and lens.max() <= 8192
    assert int(np.minimum(w.window, lens).sum()) == 65536
    w = synth.workload("same_family")
    assert w.B == 128 and (w.H_s, w.H_t, w.V) == (2560, 4096, 151936)
    assert set(np.unique(w.window)) <= {256, 512, 1024, 2048} | set(np.diff(w.offsets).tolist())
    w = synth.workload("probe_alignment")
    assert w.B == 16 and w.mode == synth.MODE_PREFIX_AND_FULL
    assert np.diff(w.offsets).min() >= 8192 and np.diff(w.offsets).max() <= 16384
    # same call, same structure
    assert np.array_equal(synth.workload("same_family").window, synth.workload("same_family").window)


def test_tensors_are_seeded_bf16_with_the_stated_scale():
    a = synth.normal_bf16((300, 64), 0.02, ("x", 1), chunk_rows=128)
    b = synth.normal_bf16((300, 64), 0.02, ("x", 1), chunk_rows=128)
    assert a.dtype == torch.bfloat16 and torch.equal(a, b)
    assert not torch.equal(a, synth.normal_bf16((300, 64), 0.02, ("x", 2)))
    assert abs(float(a.float().std()) - 0.02) < 2e-3
    f = synth.to_f64(a)
    assert f.dtype == np.float64 and np.array_equal(f.astype(np.float32), a.float().numpy())
    ids = synth.uniform_ids(1000, 77, "k")
    assert ids.dtype == torch.int32 and int(ids.min()) >= 0 and int(ids.max()) < 77


def test_sample_rows_cover_window_edges():
    w = synth.workload("strong_to_weak")
    rows = synth.sample_rows(w, 512)
    assert len(rows) <= 512 and len(np.unique(rows)) == len(rows)
    adm = set(O.plan(w.offsets, w.window)["rows"].tolist())
    assert all(int(r) in adm for r in rows)
    assert 0 in rows and int(w.offsets[1]) - 1 not in rows and 1023 in rows
    w5 = synth.workload("probe_alignment")
    rows5 = synth.sample_rows(w5, 64)
    assert 2048 in rows5 and 2047 in rows5 and int(w5.offsets[1]) - 1 in rows5


def test_tiny_config_oracle_invariants():
    w = synth.workload("tiny_probe")
    p = synth.hidden_problem(w)
    f = {k: synth.to_f64(v) for k, v in p.items() if k != "ids"}
    out = O.supervise(f["h_s"], f["h_t"], f["W_s"], f["W_t"], p["ids"].numpy(),
                      w.offsets, w.window, mode=O.MODE_PREFIX_AND_FULL)
    assert out["n"].tolist() == [64, 128] and out["n_adm"] == 192
    assert np.all(out["kl"] > 0)
    # the second rollout is fully covered by its window
    assert out["loss_prefix"][1] == out["loss_full"][1]
    assert abs(out["rho_pooled"][1] - 1) < 1e-12 and abs(out["rho_field"][1] - 1) < 1e-12
    assert 0 < out["rho_field"][0] < 1
    assert np.all(out["dh_prefix"][64:96] == 0) and np.any(out["dh_full"][64:96] != 0)
    # teacher == student gives zero loss and zero gradient
    same = O.supervise(f["h_s"], f["h_s"], f["W_s"], f["W_s"], None, w.offsets, w.window)
    assert np.all(np.abs(same["kl"]) < 1e-15) and np.all(np.abs(same["g"]) < 1e-17)
