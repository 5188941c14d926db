"""kda_chunk_fwd_static_scratch: the entry point that allocates nothing (its workspace is a static device
array inside the library) against kda_chunk_fwd on the same inputs, through the C ABI."""
import gc

import numpy as np
import pytest
import torch

import synth_inputs as si
from helpers import rel_err, to_device, oracle_prefill, worst_slice_err, o_slices, state_slices

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3    # the stated tolerance of the bf16 prefill, here between the two entry points and against the oracle


def _both(x, **kw):
    import paper_2510_26692_amd as kda
    dd = to_device(x)
    args = (dd["q"], dd["k"], dd["v"], dd["log_alpha"], dd["beta"])
    o_ref, h_ref = kda.kda_chunk_fwd(*args, h0=dd.get("h0"), cu_seqlens=dd.get("cu_seqlens"), check=True, **kw)
    o = torch.full_like(o_ref, float("nan"))
    hT = torch.full_like(h_ref, float("nan"))
    gc.collect()                                             # (garbage of earlier tests must not be freed in between)
    before = torch.cuda.memory_allocated()
    kda.kda_chunk_fwd_static_scratch(*args, o, hT=hT, h0=dd.get("h0"), cu_seqlens=dd.get("cu_seqlens"), **kw)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return o, hT, o_ref, h_ref


def test_static_scratch_entry_point_matches_kda_chunk_fwd_twice_in_a_row():
    """Two calls in a row on the shared array, the second with a smaller input: what the first call left in
    the array (slots, flags, counters) must not leak into the second.  The long input does not fit the
    64 MiB in one time segment, so the state carry between segments runs too."""
    import paper_2510_26692_amd as kda
    assert kda.kda_static_scratch_size() == 64 << 20
    big = si.make_prefill(2, 64 * 40 + 17, 8, 128, 128, "bf16", -2.0, 801, 0.02)       # 16 pairs of 41 chunks
    small = si.make_varlen([130, 0, 64, 7], 3, 128, 128, "bf16", -2.0, 802, 0.05)
    for name, x in (("big", big), ("small", small)):
        kw = {}
        o, hT, o_ref, h_ref = _both(x, **kw)
        B, T, H, _ = x["q"].shape
        cu = None if x.get("cu_seqlens") is None else x["cu_seqlens"].cpu().numpy()
        N = B if cu is None else len(cu) - 1
        e_o = worst_slice_err(o.cpu().numpy(), o_ref.cpu().numpy(), o_slices(B, H, cu))
        e_h = worst_slice_err(hT.cpu().numpy(), h_ref.cpu().numpy(), state_slices(N, H))
        oo, ho = oracle_prefill(x)
        e_oo = worst_slice_err(o.cpu().numpy(), oo, o_slices(B, H, cu))
        e_ho = worst_slice_err(hT.cpu().numpy(), ho, state_slices(N, H))
        print("static scratch %s: vs kda_chunk_fwd %.2e / %.2e, vs oracle %.2e / %.2e" % (name, e_o, e_h, e_oo, e_ho))
        assert e_o <= TOL_BF16 and e_h <= TOL_BF16 and e_oo <= TOL_BF16 and e_ho <= TOL_BF16


def test_static_scratch_entry_point_with_many_time_segments_and_fp32_inputs():
    import paper_2510_26692_amd as kda
    # 128 pairs: 64 MiB hold about six chunk indices per segment, the sequence has 12
    x = si.make_prefill(8, 64 * 12 - 5, 16, 128, 128, "bf16", -2.0, 803, 0.02)
    o, hT, o_ref, h_ref = _both(x)
    assert torch.equal(o, o_ref) and torch.equal(hT, h_ref)          # no time split with 128 pairs: same arithmetic, same bits
    y = si.make_prefill(2, 200, 2, 64, 64, "f32", -1.0, 804, 0.05)
    o, hT, o_ref, h_ref = _both(y)
    assert rel_err(o.cpu().numpy(), o_ref.cpu().numpy()) <= 2e-5 and rel_err(hT.cpu().numpy(), h_ref.cpu().numpy()) <= 2e-5


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import paper_2510_26692_amd as kda
    x = si.make_prefill(8, 256, 32, 128, 128, "bf16", -2.0, 805, 0.0)              # 256 pairs of four chunks: beyond the array
    dd = to_device(x)
    o = torch.empty(8, 256, 32, 128, device="cuda")
    with pytest.raises(kda.KdaError) as ei:
        kda.kda_chunk_fwd_static_scratch(dd["q"], dd["k"], dd["v"], dd["log_alpha"], dd["beta"], o)
    assert ei.value.status == 3 and "static array" in str(ei.value)
