"""Full-size parity runs of the baseline workloads (configs 1-3) on the GPU."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from helpers import check_prefill, o_slices, rel_err, state_slices, worst_slice_err

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3   # stated tolerance for bf16 inputs: max|x-ref|/max|ref| per (sequence, head)


def test_config1_prefill_bf16_full():
    c = si.CONFIGS["cfg1_prefill_bf16"]
    d = si.make_prefill(c["B"], c["T"], c["H"], c["dk"], c["dv"], c["dtype"], c["mu"], c["seed"],
                        c["h0_std"])
    eo, eh = check_prefill(d, TOL_BF16)
    print("config 1: err_o %.2e err_hT %.2e" % (eo, eh))


def test_config2_varlen_bf16_full():
    c = si.CONFIGS["cfg2_varlen_bf16"]
    lens = si.varlen_lengths(c["N"], c["len_lo"], c["len_hi"], c["seed"])
    d = si.make_varlen(lens, c["H"], c["dk"], c["dv"], c["dtype"], c["mu"], c["seed"], c["h0_std"])
    eo, eh = check_prefill(d, TOL_BF16, max_seqlen=int(lens.max()))
    print("config 2 (lens %s): err_o %.2e err_hT %.2e" % (lens.tolist(), eo, eh))


def test_config3_long_context_1m_tokens():
    """B=1, H=32, T=2^20.  Inputs are generated on the device.  With |k| <= 1 and beta in [0,1] every
    transition is a contraction scaled by the decay, so the state W tokens before a position influences
    it by at most exp(max_d sum log alpha) of its norm: the oracle run from a zero state over a window
    equals the full-history result on the window's tail up to that bound, which the test evaluates for
    every window and requires to be below 1e-30.  Checked that way: o on the first 16384 tokens (from
    the true zero state), h_T and o on the last 4096 tokens, and o on 4096 tokens around EVERY place
    where the call hands a state from one piece of work to another: the boundaries between time
    segments (state carry) and between the ranges of the time-split scan (folded range states).  Two
    calls: one with a workspace bounded to 1024 chunk indices per segment, one with the full
    single-segment workspace, the plan bench.py times."""
    import paper_2510_26692_amd as kda
    c = si.CONFIGS["cfg3_long_bf16"]
    T, H, dk, dv = c["T"], c["H"], c["dk"], c["dv"]
    x = si.make_long_on_device(T, H, dk, dv, c["dtype"], c["mu"], c["seed"], "cuda")
    dims = kda.kda.make_chunk_dims(x["q"], x["v"])

    def part(t0, t1):
        return [si.to_np32(x[n_][:, t0:t1]) for n_ in ("q", "k", "v", "log_alpha", "beta")]

    P = 16384
    o_prefix, _ = oracle.kda_forward(*part(0, P), want_hT=False)
    Sfx, Chk = 8192, 4096
    q_, k_, v_, g_, b_ = part(T - Sfx, T)
    bound_tail = float(np.exp(np.max(np.sum(g_[0, :Sfx - Chk].astype(np.float64), axis=0))))
    assert bound_tail < 1e-30, bound_tail
    o_sfx, h_sfx = oracle.kda_forward(q_, k_, v_, g_, b_)

    def window_error(o, b):
        """o on [b - 2048, b + 2048) against the oracle started from zero at b - 8192."""
        t0, t1 = b - 8192, min(b + 2048, T)
        qw, kw, vw, gw, bw = part(t0, t1)
        bound = float(np.exp(np.max(np.sum(gw[0, :8192 - 2048].astype(np.float64), axis=0))))
        assert bound < 1e-30, (b, bound)
        o_w, _ = oracle.kda_forward(qw, kw, vw, gw, bw, want_hT=False)
        return worst_slice_err(o[:, b - 2048:t1].cpu().numpy(), o_w[:, 8192 - 2048:], o_slices(1, H))

    full_bytes = kda.kda_chunk_fwd_workspace_size(dims)
    per_index = full_bytes // (T // 64)
    o = torch.empty(1, T, H, dv, dtype=torch.float32, device="cuda")
    hT = torch.empty(1, H, dk, dv, dtype=torch.float32, device="cuda")
    for name, ws_bytes in (("1024-chunk segments", 1024 * per_index + 64 * H * dk * dv * 4 + 8192), ("single segment", full_bytes)):
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        seg_chunks, nseg, parts, part0, part_len = kda.kda_debug_chunk_fwd_plan(dims, ws_bytes)
        o.fill_(float("nan"))
        kda.kda_chunk_fwd(x["q"], x["k"], x["v"], x["log_alpha"], x["beta"], o=o, hT=hT, workspace=ws, check=True)
        torch.cuda.synchronize()
        # chunk indices at which a state changes hands
        bounds = set()
        segs = list(range(nseg)) if nseg <= 4 else [0, 1, nseg // 2, nseg - 1]
        for sgm in segs:
            if sgm > 0:
                bounds.add(sgm * seg_chunks)
            if parts > 1:
                for p in range(1, parts):
                    bounds.add(sgm * seg_chunks + part0 + (p - 1) * part_len)
        bounds = sorted(bb for bb in bounds if 8192 // 64 <= bb < T // 64)
        assert (nseg > 1 or parts > 1) and bounds, (name, seg_chunks, nseg, parts)
        errs = [window_error(o, 64 * bb) for bb in bounds]
        e_prefix = worst_slice_err(o[:, :P].cpu().numpy(), o_prefix, o_slices(1, H))
        e_tail = worst_slice_err(o[:, T - Chk:].cpu().numpy(), o_sfx[:, Sfx - Chk:], o_slices(1, H))
        e_hT = worst_slice_err(hT.cpu().numpy(), h_sfx, state_slices(1, H))
        assert torch.isfinite(o[:, ::4097]).all()
        print("config 3, %s (%d chunks x %d segments, %d ranges of %d / %d chunks): err_o(prefix 16k) %.2e err_o(last 4k) %.2e "
              "err_hT %.2e; %d hand-over windows, worst err_o %.2e (ignored-prefix bound %.1e)"
              % (name, seg_chunks, nseg, parts, part0, part_len, e_prefix, e_tail, e_hT, len(errs), max(errs), bound_tail))
        assert e_prefix <= TOL_BF16 and e_tail <= TOL_BF16 and e_hT <= TOL_BF16
        assert max(errs) <= TOL_BF16, list(zip(bounds, errs))
        del ws
