"""Shared helpers for the parity tests: error metric and oracle plumbing."""
import numpy as np
import torch

import oracle
import synth_inputs as si


def rel_err(x, ref):
    """max|x - ref| / max|ref| over the whole array (0/0 counts as 0)."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.max(np.abs(ref)) if ref.size else 0.0
    num = np.max(np.abs(x - ref)) if ref.size else 0.0
    if den == 0.0:
        return 0.0 if num == 0.0 else np.inf
    return float(num / den)


def worst_slice_err(x, ref, seq_axis_slices):
    """The parity metric: max over (sequence, head) slices of rel_err, and over the
    whole tensor.  `seq_axis_slices` yields index tuples selecting one slice each."""
    worst = rel_err(x, ref)
    for idx in seq_axis_slices:
        worst = max(worst, rel_err(x[idx], ref[idx]))
    return worst


def o_slices(B, H, cu=None):
    if cu is None:
        return [(b, slice(None), h) for b in range(B) for h in range(H)]
    return [(0, slice(int(s), int(e)), h) for s, e in zip(cu[:-1], cu[1:]) if e > s
            for h in range(H)]


def state_slices(N, H):
    return [(n, h) for n in range(N) for h in range(H)]


def oracle_prefill(d, scale=1.0):
    """Run the fp64 oracle on a dict produced by synth_inputs (any device)."""
    cu = None if d.get("cu_seqlens") is None else d["cu_seqlens"].cpu().numpy().astype(np.int64)
    h0 = None if d.get("h0") is None else d["h0"].cpu().numpy().astype(np.float64)
    return oracle.kda_forward(si.to_np32(d["q"]), si.to_np32(d["k"]), si.to_np32(d["v"]),
                              si.to_np32(d["log_alpha"]), si.to_np32(d["beta"]), h0=h0,
                              cu_seqlens=cu, scale=scale)


def to_device(d, dev="cuda"):
    return {k: (v.to(dev) if isinstance(v, torch.Tensor) else v) for k, v in d.items()}


def check_prefill(d, tol, scale=1.0, **kw):
    """GPU chunk forward vs oracle on the same tensors; returns (err_o, err_hT)."""
    import paper_2510_26692_amd as kda
    dd = to_device(d)
    o, hT = kda.kda_chunk_fwd(dd["q"], dd["k"], dd["v"], dd["log_alpha"], dd["beta"],
                              h0=dd.get("h0"), cu_seqlens=dd.get("cu_seqlens"), scale=scale, check=True, **kw)
    torch.cuda.synchronize()
    o_ref, hT_ref = oracle_prefill(d, scale)
    B, T, H, _ = d["q"].shape
    cu = None if d.get("cu_seqlens") is None else d["cu_seqlens"].cpu().numpy()
    N = B if cu is None else len(cu) - 1
    o_np = o.cpu().numpy()
    hT_np = hT.cpu().numpy()
    assert np.isfinite(o_np).all() and np.isfinite(hT_np).all()
    eo = worst_slice_err(o_np, o_ref, o_slices(B, H, cu))
    eh = worst_slice_err(hT_np, hT_ref, state_slices(N, H))
    assert eo <= tol, "o error %.3e exceeds %.1e" % (eo, tol)
    assert eh <= tol, "hT error %.3e exceeds %.1e" % (eh, tol)
    return eo, eh
