"""The scalar-gate special case of Eq. (1) (Section 2.2: one decay per token and head) through its
own entry points: parity against the oracle, and agreement with the per-channel entry point on the
decay repeated over the channels."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from helpers import o_slices, rel_err, state_slices, to_device, worst_slice_err

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3   # stated tolerance for bf16 inputs
TOL_F32 = 1e-5


def _scalar_problem(x):
    """Same tensors with the first channel's decay taken as the head's decay."""
    y = dict(x)
    y["log_alpha_head"] = x["log_alpha"][..., 0].contiguous()
    y["log_alpha"] = y["log_alpha_head"][..., None].expand_as(x["log_alpha"]).contiguous()
    return y


def _check(x, **kw):
    import paper_2510_26692_amd as kda
    dd = to_device(x)
    o, hT = kda.kda_chunk_fwd_scalar_gate(dd["q"], dd["k"], dd["v"], dd["log_alpha_head"], dd["beta"], h0=dd.get("h0"),
                                          cu_seqlens=dd.get("cu_seqlens"), check=True, **kw)
    torch.cuda.synchronize()
    cu = None if x.get("cu_seqlens") is None else x["cu_seqlens"].cpu().numpy()
    h0 = None if x.get("h0") is None else x["h0"].numpy().astype(np.float64)
    o_ref, h_ref = oracle.kda_forward_scalar_gate(si.to_np32(x["q"]), si.to_np32(x["k"]), si.to_np32(x["v"]),
                                                  si.to_np32(x["log_alpha_head"]), si.to_np32(x["beta"]), h0=h0,
                                                  cu_seqlens=None if cu is None else cu.astype(np.int64),
                                                  scale=kw.get("scale", 1.0))
    B, T, H, _ = x["q"].shape
    N = B if cu is None else len(cu) - 1
    eo = worst_slice_err(o.float().cpu().numpy(), o_ref, o_slices(B, H, cu))
    eh = worst_slice_err(hT.cpu().numpy(), h_ref, state_slices(N, H))
    return o, hT, eo, eh


@pytest.mark.parametrize("case", ["ragged", "packed", "strong_decay", "no_decay", "long_split", "long_split_short_way"])
def test_prefill_scalar_gate(case):
    import paper_2510_26692_amd as kda
    if case == "ragged":
        x = si.make_prefill(2, 300 + 37, 4, 128, 128, "bf16", -2.0, 901, 0.02)
    elif case == "packed":
        x = si.make_varlen([70, 0, 5, 129, 64, 300], 3, 128, 128, "bf16", -2.0, 902, 0.05)
    elif case == "strong_decay":
        x = si.make_prefill(2, 200, 2, 128, 128, "bf16", -2.0, 903, 0.02)
        x["log_alpha"] = (x["log_alpha"].float() * 40.0).to(torch.bfloat16)     # decays of e^-5 per token and more
    elif case == "no_decay":
        x = si.make_prefill(1, 257, 2, 128, 128, "bf16", -2.0, 904, 0.3)
        x["log_alpha"] = torch.zeros_like(x["log_alpha"])
    elif case == "long_split":                               # slow decay, short ranges: range states through the fold
        x = si.make_prefill(1, 64 * 60 - 11, 2, 128, 128, "bf16", -6.0, 905, 0.05)
    else:                                                    # fast decay, three ranges that start from the tails before them
        x = si.make_prefill(1, 64 * 60 - 11, 2, 128, 128, "bf16", -2.0, 906, 0.05)
    x = _scalar_problem(x)
    try:
        if case.startswith("long_split"):
            kda.kda_debug_set_time_split(8 if case == "long_split" else 3)
        o, hT, eo, eh = _check(x)
        # the per-channel entry point on the repeated decay computes the same function
        dd = to_device(x)
        o2, h2 = kda.kda_chunk_fwd(dd["q"], dd["k"], dd["v"], dd["log_alpha"], dd["beta"], h0=dd.get("h0"),
                                   cu_seqlens=dd.get("cu_seqlens"), check=True)
        torch.cuda.synchronize()
    finally:
        kda.kda_debug_set_time_split(1)
    d_o = (o - o2).abs().max().item() / max(o2.abs().max().item(), 1e-30)
    d_h = (hT - h2).abs().max().item() / max(h2.abs().max().item(), 1e-30)
    print("scalar gate %s: err_o %.2e err_hT %.2e; vs per-channel path %.2e / %.2e" % (case, eo, eh, d_o, d_h))
    assert eo <= TOL_BF16 and eh <= TOL_BF16
    assert d_o <= 2 * TOL_BF16 and d_h <= 2 * TOL_BF16


def test_prefill_scalar_gate_many_pairs():
    """More (sequence, head) pairs than one batch of the grid holds."""
    x = _scalar_problem(si.make_prefill(9, 300, 8, 128, 128, "bf16", -2.0, 906, 0.02))
    _, _, eo, eh = _check(x, scale=0.5)
    assert eo <= TOL_BF16 and eh <= TOL_BF16


@pytest.mark.parametrize("dtype,tol,d", [("f32", TOL_F32, 64), ("bf16", TOL_BF16, 128)])
def test_decode_scalar_gate(dtype, tol, d):
    import paper_2510_26692_amd as kda
    N, H, Tq = 5, 3, 4
    S0 = si.make_state(N, H, d, d, 0.02, 907)
    toks = [si.make_decode_tokens(N, H, d, d, dtype, -2.0, 907, t) for t in range(Tq)]
    tok = {k_: torch.stack([t_[k_] for t_ in toks], dim=1).contiguous() for k_ in toks[0]}
    gh = tok["log_alpha"][..., 0].contiguous()
    S = S0.cuda().clone()
    o = kda.kda_recurrent_steps_pooled_scalar_gate(tok["q"].cuda(), tok["k"].cuda(), tok["v"].cuda(), gh.cuda(),
                                                   tok["beta"].cuda(), S, scale=0.9)
    torch.cuda.synchronize()
    o_ref, S_ref = oracle.kda_steps_pooled_scalar_gate(si.to_np32(tok["q"]), si.to_np32(tok["k"]), si.to_np32(tok["v"]),
                                                       si.to_np32(gh), si.to_np32(tok["beta"]),
                                                       S0.numpy().astype(np.float64), scale=0.9)
    eo = max(rel_err(o.cpu().numpy()[n, :, h], o_ref[n, :, h]) for n in range(N) for h in range(H))
    eS = max(rel_err(S.cpu().numpy()[n, h], S_ref[n, h]) for n in range(N) for h in range(H))
    print("scalar gate decode %s: err_o %.2e err_S %.2e" % (dtype, eo, eS))
    assert eo <= tol and eS <= tol


def test_scalar_gate_prefill_needs_the_matrix_core_path():
    import paper_2510_26692_amd as kda
    x = to_device(si.make_prefill(1, 64, 1, 64, 64, "f32", -2.0, 908, 0.0))
    with pytest.raises(kda.KdaError) as e:
        kda.kda_chunk_fwd_scalar_gate(x["q"], x["k"], x["v"], x["log_alpha"][..., 0].contiguous(), x["beta"])
    assert e.value.status == 2
