"""The calls are chains of kernel launches on the caller's stream (the plan made from the host
arrays travels in kernel arguments), so a caller may capture them in a HIP graph.  A captured
call must give, on every replay, exactly what an eager call gives on the inputs that are in
the buffers at that moment."""
import numpy as np
import pytest
import torch

from paper_2605_28396_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2605_28396_amd import binding
    return binding


def test_init_is_idempotent(B):
    B.adwin_opd_init()
    B.adwin_opd_init()


def _snapshot(out):
    return {k: v.clone() for k, v in out.items()}


def _replays_match_eager(call, mutate, replays=3):
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):                 # first use of the kernels happens outside the capture
        assert call.run(side) == 0
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        assert call.run(torch.cuda.current_stream()) == 0
    for k in range(replays):
        mutate(k)                                 # eager work between the replays
        torch.cuda.synchronize()
        for v in call.out.values():
            v.fill_(7)                            # a replay that does nothing would be seen
        graph.replay()
        torch.cuda.synchronize()
        got = _snapshot(call.out)
        assert call.run() == 0                    # eager, same buffers, same inputs
        torch.cuda.synchronize()
        for name, v in call.out.items():
            assert torch.equal(v, got[name]), (k, name)
        assert int(call.out["status_dev"][0]) == 0


def test_fused_call_replays_from_a_graph(B):
    w = synth.workload("ragged_small")
    p = {k: v.cuda() for k, v in synth.hidden_problem(w).items()}
    probe = synth.workload("tiny_probe")
    for wl, prob in ((w, p), (probe, {k: v.cuda() for k, v in synth.hidden_problem(probe).items()})):
        cands = [16, 64, 100] if wl.mode == synth.MODE_PREFIX_AND_FULL else None
        want = B.FusedCall.DEFAULT_OUTPUTS + ("t_logp", "t_entropy", "t_rank")
        if wl.mode == synth.MODE_PREFIX_AND_FULL:
            want = want + ("dW_prefix", "dW_full")
        call = B.FusedCall(prob["h_s"], prob["h_t"], prob["W_s"], prob["W_t"], prob["ids"], wl.offsets,
                           wl.window, mode=wl.mode, reduction=B.ADWIN_RED_SEQ_MEAN, candidates=cands,
                           want=want)
        gen = torch.Generator(device="cuda").manual_seed(5)

        def mutate(k, prob=prob, gen=gen):
            noise = torch.randn(prob["h_s"].shape, device="cuda", generator=gen)
            prob["h_s"].copy_((prob["h_s"].float() * 0.5 + noise).to(torch.bfloat16))
            prob["W_t"].mul_(-1 if k % 2 else 1)

        _replays_match_eager(call, mutate)


def test_logits_call_replays_from_a_graph(B):
    w = synth.workload("ragged_small")
    prob = {k: v.cuda() for k, v in synth.logits_problem(w).items()}
    call = B.LogitsCall(prob["z_s"], prob["z_t"], prob["ids"], w.offsets, w.window)
    gen = torch.Generator(device="cuda").manual_seed(6)

    def mutate(k):
        noise = torch.randn(prob["z_s"].shape, device="cuda", generator=gen)
        prob["z_s"].copy_((prob["z_s"].float() + noise).to(torch.bfloat16))

    _replays_match_eager(call, mutate)
