"""The prefill and the decode step under HIP graph capture: the library allocates nothing, creates no stream or
event and clears its flags with a kernel, so a call can be recorded once and replayed.  Each test replays the
graph several times on fresh input values, with eager work and synchronisations of the program between the
replays, and checks every replay against the eager call on the same values."""
import pytest
import torch

import synth_inputs as si
from helpers import to_device

pytestmark = pytest.mark.gpu


def _fresh(x, seed):
    """New values in place (same tensors, so the recorded pointers stay valid)."""
    y = si.make_prefill(*seed[0], **seed[1])
    for k_ in ("q", "k", "v", "log_alpha", "beta", "h0"):
        if x.get(k_) is not None:
            x[k_].copy_(y[k_].to(x[k_].device))


@pytest.mark.parametrize("entry", ["workspace", "static_scratch"])
def test_prefill_replayed_from_a_graph_matches_the_eager_call(entry):
    import paper_2510_26692_amd as kda
    shape = (2, 64 * 9 + 21, 4, 128, 128, "bf16", -2.0)
    x = to_device(si.make_prefill(*shape, 501, 0.02))
    args = (x["q"], x["k"], x["v"], x["log_alpha"], x["beta"])
    dims = kda.kda.make_chunk_dims(x["q"], x["v"], None, 1.0, 0)
    ws = torch.empty(kda.kda_chunk_fwd_workspace_size(dims), dtype=torch.uint8, device="cuda")
    o = torch.empty(2, shape[1], 4, 128, dtype=torch.float32, device="cuda")
    hT = torch.empty(2, 4, 128, 128, dtype=torch.float32, device="cuda")

    def call(o_, hT_):
        if entry == "workspace":
            kda.kda_chunk_fwd(*args, h0=x["h0"], o=o_, hT=hT_, workspace=ws)
        else:
            kda.kda_chunk_fwd_static_scratch(*args, o_, hT=hT_, h0=x["h0"])

    call(o, hT)                                   # first use outside the capture (per-device set-up of the library)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            call(o, hT)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    o_ref, h_ref = torch.empty_like(o), torch.empty_like(hT)
    for rep in range(4):
        _fresh(x, (shape, dict(seed=510 + rep, h0_std=0.02)))
        o.fill_(float("nan")); hT.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got_o, got_h = o.clone(), hT.clone()
        call(o_ref, h_ref)                        # eager work of the program between the replays
        torch.cuda.synchronize()
        assert torch.equal(got_o, o_ref) and torch.equal(got_h, h_ref), "replay %d differs from the eager call" % rep


def test_decode_step_replayed_from_a_graph_matches_the_eager_call():
    import paper_2510_26692_amd as kda
    N, H, d = 6, 4, 128
    names = ("q", "k", "v", "log_alpha", "beta")
    tok = {k_: v_.cuda() for k_, v_ in si.make_decode_tokens(N, H, d, d, "bf16", -2.0, 520, 0).items()}
    S = si.make_state(N, H, d, d, 0.02, 520).cuda()
    o = torch.empty(N, H, d, dtype=torch.float32, device="cuda")
    kda.kda_recurrent_step(*[tok[n_] for n_ in names], S.clone(), o=o)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            kda.kda_recurrent_step(*[tok[n_] for n_ in names], S, o=o)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    S_ref = si.make_state(N, H, d, d, 0.02, 520).cuda()
    S.copy_(S_ref)
    o_ref = torch.empty_like(o)
    for step in range(4):
        new = si.make_decode_tokens(N, H, d, d, "bf16", -2.0, 520, 1 + step)
        for n_ in names:
            tok[n_].copy_(new[n_].cuda())
        torch.cuda.synchronize()
        graph.replay()                            # advances S in place
        torch.cuda.synchronize()
        kda.kda_recurrent_step(*[tok[n_] for n_ in names], S_ref, o=o_ref)
        torch.cuda.synchronize()
        assert torch.equal(o, o_ref) and torch.equal(S, S_ref), "replay %d differs from the eager step" % step
