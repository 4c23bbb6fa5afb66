"""The measured-ceiling probes that bench.py quotes its roofline fractions beside: they must do
what they time (the copy copies) and report rates a real MI355X can have."""
import ctypes as C

import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2605_28396_amd import binding
    return binding


def test_copy_probe_copies_and_reports_a_plausible_rate(B):
    n = 1 << 26
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
    ms = C.c_float(0)
    st = B.lib.adwin_opd_ceiling_copy(int(src.data_ptr()), int(dst.data_ptr()), n, 3, None, C.byref(ms))
    assert st == 0 and torch.equal(src, dst)
    rate = B.adwin_opd_ceiling_copy()                 # GB/s over 1 GiB, read + write
    assert 1000.0 < rate < 8000.0, rate


def test_mfma_probes_stay_below_the_published_peak(B):
    const = B.adwin_opd_ceiling_mfma()
    rand = B.adwin_opd_ceiling_mfma_random()
    assert 500.0 < rand <= const * 1.05 and const < 2600.0, (const, rand)


def test_profiling_entry_points_time_the_same_call(B):
    """The *_profile variants run the same launches between HIP events: same outputs bit for
    bit, non-negative phase times, and the phases the call does not have stay zero."""
    from paper_2605_28396_amd import synth
    w = synth.workload("ragged_mid")
    p = {k: v.cuda() for k, v in synth.hidden_problem(w).items()}
    call = B.FusedCall(p["h_s"], p["h_t"], p["W_s"], p["W_t"], p["ids"], w.offsets, w.window, mode=w.mode)
    assert call.run() == 0
    torch.cuda.synchronize()
    plain = {k: v.clone() for k, v in call.out.items()}
    ph = B.adwin_opd_fused_profile(call)
    assert set(ph) == set(B.PHASE_NAMES) and all(v >= 0.0 for v in ph.values())
    assert ph["stats"] > 0.0 and ph["dz"] > 0.0 and ph["grad"] > 0.0
    for k, v in call.out.items():
        assert torch.equal(v, plain[k]), k
    lo = {k: v.cuda() for k, v in synth.logits_problem(w).items()}
    lcall = B.LogitsCall(lo["z_s"], lo["z_t"], lo["ids"], w.offsets, w.window)
    ph = B.adwin_opd_from_logits_profile(lcall)
    assert ph["stats"] > 0.0 and ph["grad"] == 0.0 and ph["dz"] == 0.0
