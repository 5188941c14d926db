"""bf16 outputs (out_dtype KDA_BF16): o is computed in fp32 and rounded to nearest even once, at
the store.  Two checks per case: the bf16 output is bit for bit the rounded fp32 output of the same
call (same kernels, same order of operations, only the store differs), and it meets the oracle
within the bf16 tolerance plus one bf16 rounding."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from helpers import o_slices, oracle_prefill, to_device, worst_slice_err

pytestmark = pytest.mark.gpu

# The stated 2e-3 is on the fp32 output.  Rounding to bf16 (8 significant bits, round to nearest even) moves a value
# x by at most 2^-8 |x| (half a unit in the last place, the unit being at most 2^-7 |x|), so element by element
#     |o_bf16 - o_ref| <= tol + 2^-8 (|o_ref| + tol),     tol = 2e-3 max|o_ref| of the (sequence, head):
# the allowance for the rounding follows each element's own size instead of the largest one's.
TOL_BF16 = 2e-3


def bf16_out_excess(o16, o_ref, slices):
    """Largest |o16 - ref| / (tol + 2^-8 (|ref| + tol)) over all elements; at most 1 when within the bound."""
    worst = 0.0
    for sl in slices:
        ref = np.asarray(o_ref[sl], dtype=np.float64)
        tol = TOL_BF16 * np.abs(ref).max()
        bound = tol + 2.0 ** -8 * (np.abs(ref) + tol)
        worst = max(worst, float((np.abs(np.asarray(o16[sl], dtype=np.float64) - ref) / bound).max()))
    return worst


def _prefill_both(x, **kw):
    import paper_2510_26692_amd as kda
    dd = to_device(x)
    args = (dd["q"], dd["k"], dd["v"], dd["log_alpha"], dd["beta"])
    common = dict(h0=dd.get("h0"), cu_seqlens=dd.get("cu_seqlens"), check=True, **kw)
    o16, h16 = kda.kda_chunk_fwd(*args, out_dtype=torch.bfloat16, **common)
    o32, h32 = kda.kda_chunk_fwd(*args, **common)
    torch.cuda.synchronize()
    assert o16.dtype == torch.bfloat16 and o32.dtype == torch.float32
    return o16, h16, o32, h32


@pytest.mark.parametrize("case", ["ragged", "packed", "time_split", "time_split_short_way", "many_pairs"])
def test_prefill_bf16_output_is_the_rounded_fp32_output(case):
    import paper_2510_26692_amd as kda
    if case == "ragged":
        x = si.make_prefill(2, 200 + 37, 4, 128, 128, "bf16", -2.0, 401, 0.02)
    elif case == "packed":
        x = si.make_varlen([70, 0, 5, 129, 64, 300], 3, 128, 128, "bf16", -2.0, 402, 0.05)
    elif case == "time_split":                               # slow decay, short ranges: range states through the fold
        x = si.make_prefill(1, 64 * 60 - 11, 2, 128, 128, "bf16", -6.0, 403, 0.05)
    elif case == "time_split_short_way":                     # fast decay, three ranges that start from the tails before them
        x = si.make_prefill(1, 64 * 60 - 11, 2, 128, 128, "bf16", -2.0, 405, 0.05)
    else:
        x = si.make_prefill(10, 150, 8, 128, 128, "bf16", -2.0, 404, 0.02)     # 80 pairs: more than one batch of the grid
    try:
        if case.startswith("time_split"):
            kda.kda_debug_set_time_split(8 if case == "time_split" else 3)   # split for sure
        o16, h16, o32, h32 = _prefill_both(x)
    finally:
        kda.kda_debug_set_time_split(1)
    assert torch.equal(o16, o32.to(torch.bfloat16))
    assert torch.equal(h16, h32)
    o_ref, _ = oracle_prefill(x)
    B, T, H, _ = x["q"].shape
    cu = None if x.get("cu_seqlens") is None else x["cu_seqlens"].cpu().numpy()
    eo = worst_slice_err(o16.float().cpu().numpy(), o_ref, o_slices(B, H, cu))
    excess = bf16_out_excess(o16.float().cpu().numpy(), o_ref, o_slices(B, H, cu))
    print("bf16 output %s: err_o %.2e, error / element-wise bound %.3f" % (case, eo, excess))
    assert excess <= 1.0


def test_prefill_bf16_output_with_the_output_gate():
    import paper_2510_26692_amd as kda
    H, d, T = 3, 128, 341
    cu = torch.tensor([0, 200, 277, 341], dtype=torch.int32)
    gen = torch.Generator().manual_seed(405)
    og = (torch.randn(1, T, H, d, generator=gen) * 1.5).to(torch.bfloat16)
    w = 1.0 + 0.3 * torch.randn(d, generator=gen)
    x = si.make_raw_tokens(1, T, H, d, d, "bf16", -2.0, 406)
    g = {k_: v_.cuda() for k_, v_ in x.items() if isinstance(v_, torch.Tensor)}
    args = [g[n_] for n_ in ("q_raw", "k_raw", "v", "gate", "beta_logit")]
    common = dict(prologue=True, out_gate=og.cuda(), norm_weight=w.cuda(), rms_eps=1e-5, cu_seqlens=cu.cuda(),
                  scale=0.5, check=True)
    o16, h16 = kda.kda_chunk_fwd_fused(*args, out_dtype=torch.bfloat16, **common)
    o32, h32 = kda.kda_chunk_fwd_fused(*args, **common)
    torch.cuda.synchronize()
    assert torch.equal(o16, o32.to(torch.bfloat16)) and torch.equal(h16, h32)


@pytest.mark.parametrize("Tq", [1, 4])
def test_decode_bf16_output_is_the_rounded_fp32_output(Tq):
    import paper_2510_26692_amd as kda
    N, H, d = 5, 4, 128
    S0 = si.make_state(N, H, d, d, 0.02, 407)
    toks = [si.make_decode_tokens(N, H, d, d, "bf16", -2.0, 407, t) for t in range(Tq)]
    tok = {k_: torch.stack([t_[k_] for t_ in toks], dim=1).contiguous().cuda() for k_ in toks[0]}
    outs = []
    for odt in (torch.bfloat16, torch.float32):
        S = S0.cuda().clone()
        if Tq == 1:
            o = kda.kda_recurrent_step(*[tok[n_][:, 0].contiguous() for n_ in ("q", "k", "v", "log_alpha", "beta")],
                                       S, scale=0.9, out_dtype=odt)
        else:
            o = kda.kda_recurrent_steps_pooled(tok["q"], tok["k"], tok["v"], tok["log_alpha"], tok["beta"], S,
                                               scale=0.9, out_dtype=odt)
        torch.cuda.synchronize()
        assert o.dtype == odt
        outs.append((o, S))
    assert torch.equal(outs[0][0], outs[1][0].to(torch.bfloat16))
    assert torch.equal(outs[0][1], outs[1][1])
    # and against the oracle
    names = ("q", "k", "v", "log_alpha", "beta")
    o_ref, _ = oracle.kda_steps_pooled(*[si.to_np32(tok[n_].cpu()) for n_ in names],
                                       S0.numpy().astype(np.float64), np.arange(N), scale=0.9)
    o_np = outs[0][0].float().cpu().numpy().reshape(N, Tq, H, d)
    err = max(np.max(np.abs(o_np[n, :, h] - o_ref[n, :, h])) / np.max(np.abs(o_ref[n, :, h]))
              for n in range(N) for h in range(H))
    excess = bf16_out_excess(o_np, o_ref, [(n, slice(None), h) for n in range(N) for h in range(H)])
    print("bf16 decode output Tq=%d: err_o %.2e, error / element-wise bound %.3f" % (Tq, err, excess))
    assert excess <= 1.0


def test_bf16_output_needs_bf16_inputs():
    import paper_2510_26692_amd as kda
    x = to_device(si.make_prefill(1, 64, 1, 64, 64, "f32", -2.0, 408, 0.0))
    with pytest.raises(kda.KdaError) as e:
        kda.kda_chunk_fwd(x["q"], x["k"], x["v"], x["log_alpha"], x["beta"], out_dtype=torch.bfloat16)
    assert e.value.status == 2
