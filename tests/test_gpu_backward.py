"""kda_chunk_bwd (gradients of Eq. (1) through the chunkwise form of Section 3.1) against the fp64
backward oracle, element by element on the same seeded inputs, through the C ABI.

Metric: max|x - ref| / max|ref| per gradient tensor, and per (sequence, head) slice.  The path is fp32
throughout (inputs bf16 or fp32, both exact in fp32), so the bound is an fp32 one: sums of up to
C + d_k = 192 products per entry, chained over at most a few dozen chunks, each term relatively
accurate to a few 2^-24, plus the hardware exp2 (about one unit in the last place): 1e-5 (the tolerance of the fp32 forward path) leaves a
factor of about seven over what is observed (1.5e-6 at worst; the test prints the figures).
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from helpers import rel_err, to_device

pytestmark = pytest.mark.gpu

TOL = 1e-5
NAMES = ["dq", "dk", "dv", "dlog_alpha", "dbeta", "dh0"]


def _grad_inputs(x, seed, with_dhT=True):
    g = torch.Generator().manual_seed(seed)
    B, T, H, dv = x["v"].shape
    dk = x["q"].shape[-1]
    N = B if x.get("cu_seqlens") is None else x["cu_seqlens"].numel() - 1
    do = torch.randn(B, T, H, dv, generator=g)
    dhT = torch.randn(N, H, dk, dv, generator=g) * 0.1 if with_dhT else None
    return do, dhT


def _run(x, do, dhT, scale=1.0, **kw):
    import paper_2510_26692_amd as kda
    dd = to_device(x)
    out = kda.kda_chunk_bwd(dd["q"], dd["k"], dd["v"], dd["log_alpha"], dd["beta"], do.cuda(),
                            dhT=None if dhT is None else dhT.cuda(), h0=dd.get("h0"),
                            cu_seqlens=dd.get("cu_seqlens"), scale=scale, **kw)
    torch.cuda.synchronize()
    cu = None if x.get("cu_seqlens") is None else x["cu_seqlens"].cpu().numpy().astype(np.int64)
    h0 = None if x.get("h0") is None else x["h0"].numpy().astype(np.float64)
    ref = oracle.kda_backward(si.to_np32(x["q"]), si.to_np32(x["k"]), si.to_np32(x["v"]),
                              si.to_np32(x["log_alpha"]), si.to_np32(x["beta"]), do.float().numpy(),
                              dhT=None if dhT is None else dhT.numpy(), h0=h0, cu_seqlens=cu, scale=scale)
    return {n: out[n].cpu().numpy() for n in NAMES}, ref, cu


def _errors(got, ref, cu, B, H):
    errs = {}
    for name in NAMES:
        a, b = got[name], ref[name]
        assert np.isfinite(a).all(), name
        worst = rel_err(a, b)
        if name != "dh0":
            if cu is None:
                slices = [(bb, slice(None), h) for bb in range(B) for h in range(H)]
            else:
                slices = [(0, slice(int(s), int(e)), h) for s, e in zip(cu[:-1], cu[1:]) if e > s for h in range(H)]
        else:
            slices = [(n, h) for n in range(a.shape[0]) for h in range(H)]
        for idx in slices:
            den = np.abs(b[idx]).max()
            if den > 1e-3 * np.abs(b).max():          # slices with a negligible gradient are covered by the tensor-wide figure
                worst = max(worst, rel_err(a[idx], b[idx]))
        errs[name] = worst
    return errs


CASES = {
    "ragged_bf16": lambda: (si.make_prefill(2, 200, 3, 128, 128, "bf16", -2.0, 1201, 0.05), 128 ** -0.5),
    "one_short_chunk": lambda: (si.make_prefill(1, 37, 2, 128, 128, "bf16", -2.0, 1202, 0.05), 1.0),
    "exact_chunks_no_h0": lambda: (si.make_prefill(1, 256, 2, 128, 128, "bf16", -2.0, 1203, 0.0), 1.0),
    "fp32_inputs_d64": lambda: (si.make_prefill(2, 150, 2, 64, 64, "f32", -2.0, 1204, 0.05), 0.125),
    "fp32_inputs_d128": lambda: (si.make_prefill(1, 131, 2, 128, 128, "f32", -1.0, 1205, 0.05), 1.0),
    "packed": lambda: (si.make_varlen([70, 0, 5, 129, 64, 300], 2, 128, 128, "bf16", -2.0, 1206, 0.05), 1.0),
    # one row that arrives as a packed batch of one sequence (cu_seqlens = [0, T]), T a multiple of the chunk or
    # not: the packed slot layout has one slot more than the plain one, and the workspace is sized for it
    "packed_single_128": lambda: (si.make_varlen([128], 2, 128, 128, "bf16", -2.0, 1211, 0.05), 1.0),
    "packed_single_130_f32": lambda: (si.make_varlen([130], 2, 64, 64, "f32", -1.0, 1212, 0.05), 0.5),
    "bf16_inputs_d64": lambda: (si.make_prefill(2, 100, 2, 64, 64, "bf16", -2.0, 1208, 0.05), 1.0),
    "slow_decay_128_chunks": lambda: (si.make_prefill(1, 64 * 128, 1, 128, 128, "bf16", -6.0, 1209, 0.3), 128 ** -0.5),
    "slow_decay_long": lambda: (si.make_prefill(1, 64 * 20 + 9, 2, 128, 128, "bf16", -6.0, 1207, 0.05), 1.0),
}


@pytest.mark.parametrize("case", sorted(CASES))
def test_backward_parity(case):
    x, scale = CASES[case]()
    do, dhT = _grad_inputs(x, 77, with_dhT=(case != "exact_chunks_no_h0"))
    got, ref, cu = _run(x, do, dhT, scale=scale)
    B, T, H, _ = x["q"].shape
    errs = _errors(got, ref, cu, B, H)
    print(case, {k: "%.2e" % v for k, v in errs.items()})
    for name, e in errs.items():
        assert e <= TOL, "%s: %s error %.3e exceeds %.1e" % (case, name, e, TOL)


def test_backward_strong_decay_stays_finite_and_close():
    """Decays of e^-5 per token and channel and more: every decay is a pairwise difference, so nothing
    overflows.  The cumulative log decay reaches a few hundred here and is held in fp32, so a decay
    factor 2^x carries a relative error of about |x| 2^-24 ln 2 (1.2e-5 at |x| = 300), whatever the
    kernel does afterwards: the bound for this case is 4e-5."""
    x = si.make_prefill(1, 200, 2, 128, 128, "bf16", -2.0, 1210, 0.05)
    x["log_alpha"] = (x["log_alpha"].float() * 40.0).to(torch.bfloat16)
    do, dhT = _grad_inputs(x, 78)
    got, ref, cu = _run(x, do, dhT)
    for name in NAMES:
        assert np.isfinite(got[name]).all()
        assert rel_err(got[name], ref[name]) <= 4e-5, name


def test_backward_packed_leaves_stray_tokens_untouched_and_handles_empty_sequences():
    import paper_2510_26692_amd as kda
    x = si.make_varlen([0, 65, 0, 3], 2, 128, 128, "bf16", -2.0, 1211, 0.05)
    B, T, H, _ = x["q"].shape
    do, dhT = _grad_inputs(x, 79)
    got, ref, cu = _run(x, do, dhT)
    np.testing.assert_array_equal(got["dh0"][0], dhT[0].numpy())
    np.testing.assert_array_equal(got["dh0"][2], dhT[2].numpy())
    for name in NAMES:
        assert rel_err(got[name], ref[name]) <= TOL, name


def test_backward_rejects_bad_calls():
    import paper_2510_26692_amd as kda
    x = to_device(si.make_prefill(1, 100, 2, 128, 128, "bf16", -2.0, 1212, 0.0))
    do = torch.randn(1, 100, 2, 128, device="cuda")
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(kda.KdaError) as e:
        kda.kda_chunk_bwd(x["q"], x["k"], x["v"], x["log_alpha"], x["beta"], do, workspace=small)
    assert e.value.status == 3


def test_backward_many_short_sequences():
    """600 packed sequences of 0..70 tokens (the slot of a chunk comes from cu_seqlens alone)."""
    rng = np.random.default_rng(1213)
    lens = [int(v) for v in rng.integers(0, 71, size=600)]
    x = si.make_varlen(lens, 1, 128, 128, "bf16", -2.0, 1213, 0.05)
    do, dhT = _grad_inputs(x, 80)
    got, ref, cu = _run(x, do, dhT, max_seqlen=70)
    for name in NAMES:
        assert rel_err(got[name], ref[name]) <= TOL, name


def test_backward_zero_tokens_and_zero_sequences():
    import paper_2510_26692_amd as kda
    z = lambda *shape, dt=torch.bfloat16: torch.zeros(*shape, dtype=dt, device="cuda")
    out = kda.kda_chunk_bwd(z(2, 0, 3, 128), z(2, 0, 3, 128), z(2, 0, 3, 128), z(2, 0, 3, 128), z(2, 0, 3),
                            z(2, 0, 3, 128, dt=torch.float32), dhT=torch.ones(2, 3, 128, 128, device="cuda"))
    torch.cuda.synchronize()
    assert out["dq"].shape == (2, 0, 3, 128)
    assert torch.equal(out["dh0"], torch.ones(2, 3, 128, 128, device="cuda"))   # no tokens: dh0 = dhT


def test_backward_cfg1_full_size():
    """The bench workload itself (B = 4, T = 4096, H = 16, d = 128, bf16 inputs, h0 present): 64 chunks per
    sequence, every gradient entry against the oracle."""
    c = si.CONFIGS["cfg1_prefill_bf16"]
    x = si.make_prefill(c["B"], c["T"], c["H"], c["dk"], c["dv"], c["dtype"], c["mu"], c["seed"], c["h0_std"])
    do, dhT = _grad_inputs(x, 81)
    got, ref, cu = _run(x, do, dhT)
    errs = _errors(got, ref, cu, c["B"], c["H"])
    print("cfg1", {k: "%.2e" % v for k, v in errs.items()})
    for name, e in errs.items():
        assert e <= TOL, "%s error %.3e exceeds %.1e" % (name, e, TOL)


@pytest.mark.parametrize("d", [64, 128])
def test_backward_takes_bf16_output_gradients(d):
    """d_o in bf16 (the dtype o may have with bf16 inputs): widened exactly, so the same bound holds
    against the oracle fed the same bf16 values."""
    x = si.make_varlen([150, 3, 64], 2, d, d, "bf16", -2.0, 1214, 0.05)
    do, dhT = _grad_inputs(x, 82)
    do = do.to(torch.bfloat16)
    got, ref, cu = _run(x, do, dhT, scale=d ** -0.5)
    for name in NAMES:
        assert rel_err(got[name], ref[name]) <= TOL, name


def test_backward_cfg2_packed_full_size_sampled_heads():
    """The packed baseline workload (8 sequences of 512..8192 tokens, 32 heads, d = 128): the GPU runs all of
    it; heads never mix, so the oracle is run on two of the 32 heads and every gradient of those is compared."""
    import paper_2510_26692_amd as kda
    c = si.CONFIGS["cfg2_varlen_bf16"]
    lens = si.varlen_lengths(c["N"], c["len_lo"], c["len_hi"], c["seed"])
    x = si.make_varlen(lens, c["H"], c["dk"], c["dv"], c["dtype"], c["mu"], c["seed"], 0.02)
    do, dhT = _grad_inputs(x, 83)
    dd = to_device(x)
    out = kda.kda_chunk_bwd(dd["q"], dd["k"], dd["v"], dd["log_alpha"], dd["beta"], do.cuda(), dhT=dhT.cuda(),
                            h0=dd["h0"], cu_seqlens=dd["cu_seqlens"], max_seqlen=int(lens.max()))
    torch.cuda.synchronize()
    heads = [3, 29]
    cu = x["cu_seqlens"].numpy().astype(np.int64)
    ref = oracle.kda_backward(si.to_np32(x["q"][:, :, heads]), si.to_np32(x["k"][:, :, heads]),
                              si.to_np32(x["v"][:, :, heads]), si.to_np32(x["log_alpha"][:, :, heads]),
                              si.to_np32(x["beta"][:, :, heads]), do[:, :, heads].numpy(),
                              dhT=dhT[:, heads].numpy(), h0=x["h0"][:, heads].numpy().astype(np.float64),
                              cu_seqlens=cu)
    for name in NAMES:
        got = out[name].cpu().numpy()
        got = got[:, heads] if name == "dh0" else got[:, :, heads]
        e = rel_err(got, ref[name])
        assert e <= TOL, "%s error %.3e exceeds %.1e" % (name, e, TOL)


def test_backward_binding_reuses_the_output_tensors_it_is_given():
    import paper_2510_26692_amd as kda
    x = to_device(si.make_prefill(1, 130, 2, 128, 128, "bf16", -2.0, 1215, 0.05))
    do = torch.randn(1, 130, 2, 128, device="cuda")
    first = kda.kda_chunk_bwd(x["q"], x["k"], x["v"], x["log_alpha"], x["beta"], do, h0=x["h0"])
    keep = {n: t.clone() for n, t in first.items()}
    ptrs = {n: t.data_ptr() for n, t in first.items()}
    for t in first.values():
        t.fill_(7.0)
    again = kda.kda_chunk_bwd(x["q"], x["k"], x["v"], x["log_alpha"], x["beta"], do, h0=x["h0"], out=first)
    torch.cuda.synchronize()
    for n in NAMES:
        assert again[n].data_ptr() == ptrs[n] and torch.equal(again[n], keep[n]), n
    with pytest.raises(ValueError):
        kda.kda_chunk_bwd(x["q"], x["k"], x["v"], x["log_alpha"], x["beta"], do, h0=x["h0"],
                          out={**first, "dq": first["dq"][:, :64]})
