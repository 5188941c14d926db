"""GPU parity of kda_recurrent_step against the fp64 oracle (Eq. (1), one token)."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from helpers import rel_err, state_slices, worst_slice_err

pytestmark = pytest.mark.gpu

# fp32 arithmetic on both the state and the token vectors: the only differences
# from the fp64 oracle are fp32 rounding of ~dk products per output and the
# hardware exp2 (1 ulp), so errors sit near 1e-6; the gate is the stated one.
TOL_F32 = 1e-5
TOL_BF16 = 2e-3


def _run_steps(N, H, d, dtype, steps, seed, scale=1.0):
    import paper_2510_26692_amd as kda
    S0 = si.make_state(N, H, d, d, 0.02, seed)
    S_gpu = S0.cuda().clone()
    S_ref = S0.numpy().astype(np.float64)
    worst_o = 0.0
    for s in range(steps):
        tok = si.make_decode_tokens(N, H, d, d, dtype, -2.0, seed, s)
        g = {k_: v_.cuda() for k_, v_ in tok.items()}
        o = kda.kda_recurrent_step(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], S_gpu, scale=scale)
        o_ref, S_ref = oracle.kda_step(si.to_np32(tok["q"]), si.to_np32(tok["k"]), si.to_np32(tok["v"]),
                                       si.to_np32(tok["log_alpha"]), si.to_np32(tok["beta"]), S_ref,
                                       scale=scale)
        worst_o = max(worst_o, worst_slice_err(o.cpu().numpy(), o_ref, state_slices(N, H)))
    torch.cuda.synchronize()
    err_S = worst_slice_err(S_gpu.cpu().numpy(), S_ref, state_slices(N, H))
    return worst_o, err_S


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("dtype,tol", [("f32", TOL_F32), ("bf16", TOL_BF16)])
def test_decode_small(d, dtype, tol):
    eo, eS = _run_steps(N=3, H=5, d=d, dtype=dtype, steps=7, seed=11, scale=0.7)
    print("decode d=%d %s: err_o %.2e err_S %.2e" % (d, dtype, eo, eS))
    assert eo <= tol and eS <= tol


def test_decode_config4_full_size_100_steps():
    """256 sequences x 32 heads, 128x128 fp32 states (512 MiB), 100 steps with fresh
    bf16 tokens; the state after the last step and the last o are checked."""
    import paper_2510_26692_amd as kda
    cfg = si.CONFIGS["cfg4_decode_bf16"]
    N, H, d, steps = cfg["N"], cfg["H"], cfg["dk"], cfg["steps"]
    S0 = si.make_state(N, H, d, d, cfg["state_std"], cfg["seed"])
    S_gpu = S0.cuda().clone()
    S_ref = S0.numpy().astype(np.float64)
    for s in range(steps):
        tok = si.make_decode_tokens(N, H, d, d, cfg["dtype"], cfg["mu"], cfg["seed"], s)
        g = {k_: v_.cuda() for k_, v_ in tok.items()}
        o = kda.kda_recurrent_step(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], S_gpu)
        o_ref, S_ref = oracle.kda_step(si.to_np32(tok["q"]), si.to_np32(tok["k"]), si.to_np32(tok["v"]),
                                       si.to_np32(tok["log_alpha"]), si.to_np32(tok["beta"]), S_ref)
    torch.cuda.synchronize()
    eS = worst_slice_err(S_gpu.cpu().numpy(), S_ref, state_slices(N, H))
    eo = worst_slice_err(o.cpu().numpy(), o_ref, state_slices(N, H))
    print("config 4: err_S %.2e err_o(last) %.2e" % (eS, eo))
    assert eS <= TOL_BF16 and eo <= TOL_BF16


def test_decode_rejects_bad_arguments():
    import paper_2510_26692_amd as kda
    q = torch.zeros(2, 2, 128, device="cuda")
    S = torch.zeros(2, 2, 128, 128, device="cuda")
    b = torch.zeros(2, 2, device="cuda")
    with pytest.raises(ValueError):
        kda.kda_recurrent_step(q, q, q, q, b, S[:, :, :64])
    q96 = torch.zeros(2, 2, 96, device="cuda")
    S96 = torch.zeros(2, 2, 96, 96, device="cuda")
    with pytest.raises(kda.KdaError) as ei:
        kda.kda_recurrent_step(q96, q96, q96, q96, b, S96)
    assert ei.value.status == 2


def _stack_tokens(N, H, d, dtype, Tq, seed):
    toks = [si.make_decode_tokens(N, H, d, d, dtype, -2.0, seed, t) for t in range(Tq)]
    return {k_: torch.stack([t_[k_] for t_ in toks], dim=1).contiguous() for k_ in toks[0]}


@pytest.mark.parametrize("Tq", [1, 3, 8])
@pytest.mark.parametrize("dtype,tol,d", [("f32", TOL_F32, 64), ("bf16", TOL_BF16, 128)])
def test_pooled_multi_token_decode(Tq, dtype, tol, d):
    """Sequences name states of a larger pool through a permuted index array with skipped entries;
    each takes Tq tokens through its state in one call.  Checked against the oracle: o, the named
    states, and that every other state of the pool is bit-for-bit untouched."""
    import paper_2510_26692_amd as kda
    N, H, P = 6, 4, 11
    pool0 = si.make_state(P, H, d, d, 0.02, 31)
    idx = torch.tensor([7, 2, -1, 10, 0, 5], dtype=torch.int32)
    tok = _stack_tokens(N, H, d, dtype, Tq, 31)
    g = {k_: v_.cuda() for k_, v_ in tok.items()}
    pool = pool0.cuda().clone()
    o_init = torch.full((N, Tq, H, d), 7.0, device="cuda")
    o = kda.kda_recurrent_steps_pooled(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], pool, idx.cuda(),
                                       scale=0.9, o=o_init)
    torch.cuda.synchronize()
    o_ref, pool_ref = oracle.kda_steps_pooled(si.to_np32(tok["q"]), si.to_np32(tok["k"]), si.to_np32(tok["v"]),
                                              si.to_np32(tok["log_alpha"]), si.to_np32(tok["beta"]),
                                              pool0.numpy().astype(np.float64), idx.numpy(), scale=0.9)
    o_np, pool_np = o.cpu().numpy(), pool.cpu().numpy()
    act = [n for n in range(N) if idx[n] >= 0]
    eo = max(rel_err(o_np[n, :, h], o_ref[n, :, h]) for n in act for h in range(H))
    eS = max(rel_err(pool_np[int(idx[n]), h], pool_ref[int(idx[n]), h]) for n in act for h in range(H))
    print("pooled decode Tq=%d %s: err_o %.2e err_S %.2e" % (Tq, dtype, eo, eS))
    assert eo <= tol and eS <= tol
    assert (o_np[2] == 7.0).all()                                   # skipped sequence: o untouched
    unused = [p_ for p_ in range(P) if p_ not in idx.tolist()]
    assert torch.equal(pool.cpu()[unused], pool0[unused])            # states nobody named


def test_pooled_decode_without_indices_equals_the_plain_step_and_rejects_bad_sizes():
    import paper_2510_26692_amd as kda
    N, H, d = 3, 2, 128
    S0 = si.make_state(N, H, d, d, 0.02, 41)
    tok = si.make_decode_tokens(N, H, d, d, "bf16", -2.0, 41, 0)
    g = {k_: v_.cuda() for k_, v_ in tok.items()}
    S1, S2 = S0.cuda().clone(), S0.cuda().clone()
    o1 = kda.kda_recurrent_step(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], S1)
    o2 = kda.kda_recurrent_steps_pooled(g["q"][:, None].contiguous(), g["k"][:, None].contiguous(),
                                        g["v"][:, None].contiguous(), g["log_alpha"][:, None].contiguous(),
                                        g["beta"][:, None].contiguous(), S2)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2[:, 0]) and torch.equal(S1, S2)
    big = _stack_tokens(N, H, d, "bf16", 9, 41)
    gb = {k_: v_.cuda() for k_, v_ in big.items()}
    with pytest.raises(kda.KdaError) as ei:
        kda.kda_recurrent_steps_pooled(gb["q"], gb["k"], gb["v"], gb["log_alpha"], gb["beta"], S2)
    assert ei.value.status == 1
