"""The entry point that allocates nothing (adwin_opd_from_logits_static): called through the
C ABI, its outputs must equal those of adwin_opd_from_logits bit for bit (same kernels, the
scratch in the library's static array instead of a caller workspace), on two calls in a row, the
second on a smaller problem, and an over-sized problem must be refused."""
import ctypes as C

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


def _bits(t):
    return t.view(torch.int16) if t.dtype == torch.bfloat16 else t


def _both(B, w, p, **kw):
    d = {k: v.cuda() for k, v in p.items()}
    want = ("kl", "c", "dz", "loss_prefix", "batch", "n_out", "n_adm_out", "status_dev",
            "t_logp", "t_entropy", "t_rank", "t_first_reject", "t_logp_mean")
    ref = B.LogitsCall(d["z_s"], d["z_t"], d["ids"], w.offsets, w.window, want=want, topk=100, **kw)
    new = B.LogitsCall(d["z_s"], d["z_t"], d["ids"], w.offsets, w.window, want=want, topk=100,
                       workspace=False, **kw)
    assert new.workspace is None
    for t in new.out.values():          # whatever the outputs hold before the call must not survive it
        t.view(torch.uint8).fill_(0xA5)
    assert ref.run() == 0
    before = torch.cuda.memory_allocated()
    assert new.run_static() == 0
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for k in want:
        assert torch.equal(_bits(new.out[k]), _bits(ref.out[k])), k
    return {k: (v.float() if v.dtype.is_floating_point else v).cpu().numpy() for k, v in new.out.items()}, d


def test_static_scratch_entry_point_matches_the_workspace_one(B):
    # first call: several rollouts, windows ending inside, at and beyond them
    w1 = synth.workload("ragged_mid")
    p1 = synth.logits_problem(w1)
    got1, _ = _both(B, w1, p1, reduction=O.RED_SEQ_MEAN, grad_scale=2.0)
    # second call, smaller input (fewer rows, fewer rollouts, smaller vocabulary): the array still
    # holds the first call's plan and sums, none of which may be read
    w2 = synth.workload("ragged_small")
    p2 = synth.logits_problem(w2)
    got2, _ = _both(B, w2, p2, reduction=O.RED_SUM, estimator=B.ADWIN_EST_SAMPLED)
    # and both agree with the oracle (the bar of the other parity tests)
    for w, p, got, red, est, gs in ((w1, p1, got1, O.RED_SEQ_MEAN, O.EST_EXPECTED, 2.0),
                                    (w2, p2, got2, O.RED_SUM, O.EST_SAMPLED, 1.0)):
        f = Hp.oracle_inputs(p)
        ref = O.supervise_from_logits(f["z_s"], f["z_t"], f["ids"], w.offsets, w.window, reduction=red,
                                      grad_scale=gs, estimator=est)
        assert np.array_equal(got["n_out"], ref["n"]) and int(got["n_adm_out"][0]) == ref["n_adm"]
        assert int(got["status_dev"][0]) == 0
        Hp.assert_kl(got["kl"], ref["kl"])
        Hp.assert_cost(got["c"], ref["c"])
        Hp.assert_grad(got["dz"], ref["dz"], "dz", Hp.BF16_ULP)
        Hp.assert_close_rel(got["loss_prefix"], ref["loss_prefix"], Hp.LOSS_REL, "loss_prefix")
        Hp.assert_close_rel(got["batch"][:1], ref["batch"][:1], Hp.LOSS_REL, "L^p")
    # a third call on the first problem again, through the row-resident kernel's other scheme
    _both(B, w1, p1, reduction=O.RED_TOKEN_MEAN, scheme=B.ADWIN_LOGITS_STREAMING)


def test_static_scratch_entry_point_refuses_what_does_not_fit(B):
    """More rows than the static array has room for (4 bytes per row plus the plan): refused with
    ADWIN_E_WORKSPACE before anything is enqueued or any pointer is touched."""
    T = 300000
    off = np.array([0, T], np.int64); win = np.array([5], np.int32)
    lp = B.adwin_opd_logits_problem()
    lp.struct_bytes = C.sizeof(B.adwin_opd_logits_problem)
    lp.T, lp.B, lp.V = T, 1, 4096
    lp.offsets, lp.window = off.ctypes.data, win.ctypes.data
    lp.z_s = lp.z_t = 4096                       # never dereferenced
    assert B.adwin_opd_logits_workspace_bytes(lp) > B.ADWIN_STATIC_SCRATCH_BYTES
    assert B.lib.adwin_opd_from_logits_static(C.byref(lp), None) == B.ADWIN_E_WORKSPACE
    lp.V = 4095
    assert B.lib.adwin_opd_from_logits_static(C.byref(lp), None) == B.ADWIN_E_SHAPE
    assert B.lib.adwin_opd_from_logits_static(None, None) == B.ADWIN_E_NULL
    # the largest batch that fits is accepted by the size check (rejected later only for its
    # NULL inputs): 32 rollouts of 8,000 rows
    off = np.arange(33, dtype=np.int64) * 8000; win = np.full(32, 64, np.int32)
    lp.T, lp.B, lp.V = int(off[-1]), 32, 4096
    lp.offsets, lp.window = off.ctypes.data, win.ctypes.data
    lp.z_s = lp.z_t = None
    assert B.adwin_opd_logits_workspace_bytes(lp) <= B.ADWIN_STATIC_SCRATCH_BYTES
    assert B.lib.adwin_opd_from_logits_static(C.byref(lp), None) == B.ADWIN_E_NULL
