"""GPU parity of the fused stages of Section 4 against the fp64 oracle, for the prefill and the
pooled decode: the input prologue (L2Norm of q and k, Sigmoid of beta, decay function on the gate
logits) and the output gate (Sigmoid(gate) * head-wise RMSNorm(o))."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from helpers import gated_error_ratio, o_slices, rel_err, state_slices, worst_slice_err

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3   # stated tolerance for bf16 inputs
TOL_F32 = 1e-5
# After the output gate every token's o is divided by its own RMS, so a single max-relative number over the
# tensor no longer measures what the stated tolerance is about: the gated tests check every element against
# the stated 2e-3 carried through the gate (helpers.gated_error_ratio, at most 1), and the plain metric, which
# tokens with a small o dominate, against the stated figure itself (measured 6e-4 ... 1.1e-3).
TOL_GATED_BF16 = 2e-3


def _np(d, *names):
    return [si.to_np32(d[n_]) for n_ in names]


@pytest.mark.parametrize("with_consts", [False, True])
@pytest.mark.parametrize("T", [130, 1000])
def test_prefill_fused_prologue(T, with_consts):
    import paper_2510_26692_amd as kda
    B, H, d = 2, 4, 128
    x = si.make_raw_tokens(B, T, H, d, d, "bf16", -2.0, 61 + T)
    h0 = si.make_state(B, H, d, d, 0.02, 61)
    a_scale, dt_bias = (x["a_scale"], x["dt_bias"]) if with_consts else (None, None)
    g = {k_: v_.cuda() for k_, v_ in x.items()}
    o, hT = kda.kda_chunk_fwd_fused(g["q_raw"], g["k_raw"], g["v"], g["gate"], g["beta_logit"], l2norm_eps=1e-6,
                                    a_scale=g["a_scale"] if with_consts else None,
                                    dt_bias=g["dt_bias"] if with_consts else None, h0=h0.cuda(), scale=0.8,
                                    check=True)
    torch.cuda.synchronize()
    o_ref, h_ref = oracle.kda_forward_raw(*_np(x, "q_raw", "k_raw", "v", "gate", "beta_logit"), eps=1e-6,
                                          a_scale=None if a_scale is None else a_scale.numpy(),
                                          dt_bias=None if dt_bias is None else dt_bias.numpy(),
                                          h0=h0.numpy().astype(np.float64), scale=0.8)
    eo = worst_slice_err(o.cpu().numpy(), o_ref, o_slices(B, H))
    eh = worst_slice_err(hT.cpu().numpy(), h_ref, state_slices(B, H))
    print("fused prologue prefill T=%d consts=%s: err_o %.2e err_hT %.2e" % (T, with_consts, eo, eh))
    assert eo <= TOL_BF16 and eh <= TOL_BF16


def test_prefill_fused_prologue_packed_with_short_tail():
    """Packed sequences whose last chunks are short: padding tokens must stay identity
    transitions although a zero gate logit alone would mean alpha = 1/2."""
    import paper_2510_26692_amd as kda
    lens = np.array([70, 0, 129, 5])
    H, d = 2, 128
    T = int(lens.sum())
    x = si.make_raw_tokens(1, T, H, d, d, "bf16", -1.0, 67)
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32)
    g = {k_: v_.cuda() for k_, v_ in x.items()}
    o, hT = kda.kda_chunk_fwd_fused(g["q_raw"], g["k_raw"], g["v"], g["gate"], g["beta_logit"],
                                    a_scale=g["a_scale"], dt_bias=g["dt_bias"], cu_seqlens=cu.cuda(), check=True)
    torch.cuda.synchronize()
    o_ref, h_ref = oracle.kda_forward_raw(*_np(x, "q_raw", "k_raw", "v", "gate", "beta_logit"),
                                          a_scale=x["a_scale"].numpy(), dt_bias=x["dt_bias"].numpy(),
                                          cu_seqlens=cu.numpy().astype(np.int64))
    eo = worst_slice_err(o.cpu().numpy(), o_ref, o_slices(1, H, cu.numpy()))
    eh = worst_slice_err(hT.cpu().numpy(), h_ref, state_slices(len(lens), H))
    print("fused prologue packed: err_o %.2e err_hT %.2e" % (eo, eh))
    assert eo <= TOL_BF16 and eh <= TOL_BF16
    assert (hT[1] == 0).all()                                       # empty sequence, zero initial state


@pytest.mark.parametrize("dtype,tol,d", [("f32", TOL_F32, 64), ("bf16", TOL_BF16, 128)])
def test_decode_fused_prologue(dtype, tol, d):
    import paper_2510_26692_amd as kda
    N, Tq, H, P = 5, 3, 4, 8
    x = si.make_raw_tokens(N, Tq, H, d, d, dtype, -2.0, 71)
    pool0 = si.make_state(P, H, d, d, 0.02, 71)
    idx = torch.tensor([6, 1, -1, 0, 3], dtype=torch.int32)
    g = {k_: v_.cuda() for k_, v_ in x.items()}
    pool = pool0.cuda().clone()
    o = kda.kda_recurrent_steps_fused(g["q_raw"], g["k_raw"], g["v"], g["gate"], g["beta_logit"], pool, idx.cuda(),
                                      l2norm_eps=1e-6, a_scale=g["a_scale"], dt_bias=g["dt_bias"], scale=1.1)
    torch.cuda.synchronize()
    q, k, la, b = oracle.prologue.apply(*_np(x, "q_raw", "k_raw", "gate", "beta_logit"), eps=1e-6,
                                        a_scale=x["a_scale"].numpy(), dt_bias=x["dt_bias"].numpy())
    o_ref, pool_ref = oracle.kda_steps_pooled(q, k, si.to_np32(x["v"]), la, b, pool0.numpy().astype(np.float64),
                                              idx.numpy(), scale=1.1)
    act = [n for n in range(N) if idx[n] >= 0]
    o_np, pool_np = o.cpu().numpy(), pool.cpu().numpy()
    eo = max(rel_err(o_np[n, :, h], o_ref[n, :, h]) for n in act for h in range(H))
    eS = max(rel_err(pool_np[int(idx[n]), h], pool_ref[int(idx[n]), h]) for n in act for h in range(H))
    print("fused prologue decode %s: err_o %.2e err_S %.2e" % (dtype, eo, eS))
    assert eo <= tol and eS <= tol


def test_fused_prologue_rejects_what_it_is_not_built_for():
    import paper_2510_26692_amd as kda
    x = si.make_raw_tokens(1, 64, 2, 64, 64, "f32", -2.0, 73)
    g = {k_: v_.cuda() for k_, v_ in x.items()}
    with pytest.raises(kda.KdaError) as ei:
        kda.kda_chunk_fwd_fused(g["q_raw"], g["k_raw"], g["v"], g["gate"], g["beta_logit"])
    assert ei.value.status == 2
    with pytest.raises(kda.KdaError) as ei:
        kda.kda_chunk_fwd_fused(g["q_raw"], g["k_raw"], g["v"], g["gate"], g["beta_logit"], l2norm_eps=-1.0)
    assert ei.value.status == 1


def _out_gate(shape, dtype, seed):
    gen = torch.Generator().manual_seed(seed)
    g = torch.randn(*shape, generator=gen) * 1.5
    w = 1.0 + 0.3 * torch.randn(shape[-1], generator=gen)
    return g.to(si.torch_dtype(dtype)), w


@pytest.mark.parametrize("prologue", [False, True])
def test_prefill_output_gate(prologue):
    """Output gate on top of the plain inputs (prologue off) and of the raw ones (both fused);
    packed batch with a short tail, so the per-token mean square also meets padded rows."""
    import paper_2510_26692_amd as kda
    lens = np.array([200, 77, 64])
    H, d, T = 3, 128, 341
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32)
    og, w = _out_gate((1, T, H, d), "bf16", 81)
    if prologue:
        x = si.make_raw_tokens(1, T, H, d, d, "bf16", -2.0, 83)
        names = ("q_raw", "k_raw", "v", "gate", "beta_logit")
        o_plain, h_ref = oracle.kda_forward_raw(*_np(x, *names), cu_seqlens=cu.numpy().astype(np.int64), scale=0.5)
    else:
        x = si.make_tokens(1, T, H, d, d, "bf16", -2.0, 83)
        names = ("q", "k", "v", "log_alpha", "beta")
        o_plain, h_ref = oracle.kda_forward(*_np(x, *names), cu_seqlens=cu.numpy().astype(np.int64), scale=0.5)
    g = {k_: v_.cuda() for k_, v_ in x.items() if isinstance(v_, torch.Tensor)}
    o, hT = kda.kda_chunk_fwd_fused(*[g[n_] for n_ in names], prologue=prologue, out_gate=og.cuda(),
                                    norm_weight=w.cuda(), rms_eps=1e-5, cu_seqlens=cu.cuda(), scale=0.5, check=True)
    torch.cuda.synchronize()
    o_ref = oracle.epilogue.apply(o_plain, si.to_np32(og), w.numpy(), 1e-5)
    eo = worst_slice_err(o.cpu().numpy(), o_ref, o_slices(1, H, cu.numpy()))
    eh = worst_slice_err(hT.cpu().numpy(), h_ref, state_slices(len(lens), H))
    ratio = gated_error_ratio(o.cpu().numpy(), o_plain, si.to_np32(og), w.numpy(), 1e-5, o_slices(1, H, cu.numpy()), TOL_BF16)
    print("output gate prefill prologue=%s: err_o %.2e err_hT %.2e, error / carried tolerance %.3f" % (prologue, eo, eh, ratio))
    assert ratio <= 1.0 and eo <= TOL_GATED_BF16 and eh <= TOL_BF16


@pytest.mark.parametrize("dtype,tol,d", [("f32", TOL_F32, 64), ("bf16", TOL_BF16, 128)])
def test_decode_output_gate(dtype, tol, d):
    import paper_2510_26692_amd as kda
    N, Tq, H = 4, 2, 3
    toks = [si.make_decode_tokens(N, H, d, d, dtype, -2.0, 91, t) for t in range(Tq)]
    x = {k_: torch.stack([t_[k_] for t_ in toks], dim=1).contiguous() for k_ in toks[0]}
    og, w = _out_gate((N, Tq, H, d), dtype, 93)
    S0 = si.make_state(N, H, d, d, 0.02, 91)
    g = {k_: v_.cuda() for k_, v_ in x.items()}
    S = S0.cuda().clone()
    o = kda.kda_recurrent_steps_fused(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], S, prologue=False,
                                      out_gate=og.cuda(), norm_weight=w.cuda(), rms_eps=1e-5, scale=0.7)
    torch.cuda.synchronize()
    o_plain, S_ref = oracle.kda_steps_pooled(*_np(x, "q", "k", "v", "log_alpha", "beta"),
                                             S0.numpy().astype(np.float64), scale=0.7)
    o_ref = oracle.epilogue.apply(o_plain, si.to_np32(og), w.numpy(), 1e-5)
    eo = worst_slice_err(o.cpu().numpy(), o_ref, [(n, slice(None), h) for n in range(N) for h in range(H)])
    eS = worst_slice_err(S.cpu().numpy(), S_ref, state_slices(N, H))
    print("output gate decode %s: err_o %.2e err_S %.2e" % (dtype, eo, eS))
    assert eo <= tol and eS <= tol


@pytest.mark.parametrize("mu,split", [(-6.0, 8), (-2.0, 3)])
def test_prefill_output_gate_on_a_long_sequence_with_few_pairs(mu, split):
    """Few pairs and a long sequence: the time axis is cut into ranges walked side by side, and the passes that
    write outputs apply the gate; against the oracle, and against the same call with the split switched off.
    Slow decay in many short ranges (range states through the fold), and fast decay in three ranges that start
    from the tails of the ranges before them."""
    import paper_2510_26692_amd as kda
    H, d, T = 2, 128, 64 * 60 - 11
    og, w = _out_gate((1, T, H, d), "bf16", 91)
    x = si.make_tokens(1, T, H, d, d, "bf16", mu, 93)
    names = ("q", "k", "v", "log_alpha", "beta")
    o_plain, h_ref = oracle.kda_forward(*_np(x, *names), scale=0.5)
    o_ref = oracle.epilogue.apply(o_plain, si.to_np32(og), w.numpy(), 1e-5)
    g = {k_: v_.cuda() for k_, v_ in x.items() if isinstance(v_, torch.Tensor)}
    outs, parts = [], []
    try:
        for mode in (split, 0):
            kda.kda_debug_set_time_split(mode)
            dims = kda.kda.make_chunk_dims(g["q"], g["v"], None, 0.5, 0)
            parts.append(kda.kda_debug_chunk_fwd_plan(dims, 1 << 40, True)[2])
            outs.append(kda.kda_chunk_fwd_fused(*[g[n_] for n_ in names], prologue=False, out_gate=og.cuda(),
                                                norm_weight=w.cuda(), rms_eps=1e-5, scale=0.5, check=True))
        torch.cuda.synchronize()
    finally:
        kda.kda_debug_set_time_split(1)
    assert parts[0] > 1 and parts[1] == 1, parts
    for (o, hT), what in zip(outs, ("split", "one workgroup per pair")):
        eo = worst_slice_err(o.cpu().numpy(), o_ref, o_slices(1, H))
        eh = worst_slice_err(hT.cpu().numpy(), h_ref, state_slices(1, H))
        ratio = gated_error_ratio(o.cpu().numpy(), o_plain, si.to_np32(og), w.numpy(), 1e-5, o_slices(1, H), TOL_BF16)
        print("output gate, long sequence, %s (%d ranges): err_o %.2e err_hT %.2e, error / carried tolerance %.3f"
              % (what, parts[0] if what == "split" else 1, eo, eh, ratio))
        assert ratio <= 1.0 and eo <= TOL_GATED_BF16 and eh <= TOL_BF16
    # the two agree within rounding (the split forms the range states in another order)
    assert rel_err(outs[0][0].cpu().numpy(), outs[1][0].cpu().numpy()) <= TOL_BF16
