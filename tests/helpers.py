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


def gated_error_ratio(o_gated, o_plain_ref, gate, weight, eps, slices, tol):
    """Largest |o_gated - ref| / bound over all elements of the output gate's result.

    The stated tolerance is on o as the recurrence produces it: |o - o_ref| <= tol * max|o_ref| over a
    (sequence, head).  The gate (Section 4) then divides token t by r_t = sqrt(mean_j o_tj^2 + eps) and scales
    column j by w_j Sigmoid(g_tj).  To first order an error delta in o_t moves o_tj / r_t by
    delta_j / r_t - o_tj (o_t . delta) / (d r_t^3), at most |delta|_inf (1 + |o_tj| / r_t) / r_t
    (since |o_t|_1 <= d r_t), so the same tolerance carried through the gate is, per element,

        bound_tj = tol * max|o_ref| * (1 + |o_tj| / r_t) / r_t * |w_j| Sigmoid(g_tj).

    A token whose o is small next to the largest of its sequence carries the error at that larger relative size;
    the bound follows it, which one number for the whole tensor cannot."""
    o_plain_ref = np.asarray(o_plain_ref, dtype=np.float64)
    g = np.asarray(gate, dtype=np.float64)
    w = np.ones(o_plain_ref.shape[-1]) if weight is None else np.asarray(weight, dtype=np.float64)
    ref = o_plain_ref / np.sqrt(np.mean(o_plain_ref ** 2, axis=-1, keepdims=True) + eps) * w / (1.0 + np.exp(-g))
    worst = 0.0
    for sl in slices:
        op = o_plain_ref[sl]                                   # [tokens, dv]
        r = np.sqrt(np.mean(op ** 2, axis=-1, keepdims=True) + eps)
        bound = tol * np.abs(op).max() * (1.0 + np.abs(op) / r) / r * np.abs(w) / (1.0 + np.exp(-g[sl]))
        err = np.abs(np.asarray(o_gated[sl], dtype=np.float64) - ref[sl])
        worst = max(worst, float((err / np.maximum(bound, 1e-300)).max()))
    return worst


def oracle_prefill(d, scale=1.0):
    """Run the fp64 oracle on a dict produced by synth_inputs (any device)."""
    cu = None if d.get("cu_seqlens") is None else d["cu_seqlens"].cpu().numpy().astype(np.int64)
    h0 = None if d.get("h0") is None else d["h0"].cpu().numpy().astype(np.float64)
    return oracle.kda_forward(si.to_np32(d["q"]), si.to_np32(d["k"]), si.to_np32(d["v"]),
                              si.to_np32(d["log_alpha"]), si.to_np32(d["beta"]), h0=h0,
                              cu_seqlens=cu, scale=scale)


def to_device(d, dev="cuda"):
    return {k: (v.to(dev) if isinstance(v, torch.Tensor) else v) for k, v in d.items()}


GUARD_BYTES = 4096
GUARD_FILL = 0xA5


class Guarded:
    """A device tensor carved out of a larger byte buffer, with GUARD_BYTES of a known pattern on
    both sides: a kernel that writes past either end of the tensor changes the pattern."""

    def __init__(self, shape, dtype, device="cuda", fill=None):
        numel = 1
        for s_ in shape:
            numel *= int(s_)
        nbytes = numel * torch.empty((), dtype=dtype).element_size()
        self.body = (nbytes + 255) // 256 * 256
        self.nbytes = nbytes
        self.raw = torch.full((2 * GUARD_BYTES + self.body,), GUARD_FILL, dtype=torch.uint8, device=device)
        self.tensor = self.raw[GUARD_BYTES:GUARD_BYTES + nbytes].view(dtype).view(*shape)
        if fill is not None:
            self.tensor.fill_(fill)

    def assert_untouched(self, what):
        torch.cuda.synchronize()
        front = self.raw[:GUARD_BYTES]
        back = self.raw[GUARD_BYTES + self.nbytes:]
        assert bool((front == GUARD_FILL).all()), "bytes in front of %s were overwritten" % what
        assert bool((back == GUARD_FILL).all()), "bytes behind %s were overwritten" % what


def check_prefill(d, tol, scale=1.0, **kw):
    """GPU chunk forward vs oracle on the same tensors; returns (err_o, err_hT).  o, hT and (unless the
    caller brings one) the workspace sit between guard regions that must come back untouched."""
    import paper_2510_26692_amd as kda
    dd = to_device(d)
    B, T, H, _ = d["q"].shape
    dv = d["v"].shape[-1]
    N = B if dd.get("cu_seqlens") is None else dd["cu_seqlens"].numel() - 1
    guards = {}
    if "o" not in kw:
        guards["o"] = Guarded((B, T, H, dv), kw.get("out_dtype") or torch.float32, fill=0)
        kw["o"] = guards["o"].tensor
    if "hT" not in kw and kw.get("want_hT", True):
        guards["hT"] = Guarded((N, H, d["q"].shape[-1], dv), torch.float32)
        kw["hT"] = guards["hT"].tensor
    if "workspace" not in kw:
        dims = kda.kda.make_chunk_dims(dd["q"], dd["v"], dd.get("cu_seqlens"), scale, kw.get("max_seqlen", 0),
                                       kw["o"].dtype)
        need = kda.kda_chunk_fwd_workspace_size(dims)
        if need:
            guards["workspace"] = Guarded((need,), torch.uint8)
            kw["workspace"] = guards["workspace"].tensor
    o, hT = kda.kda_chunk_fwd(dd["q"], dd["k"], dd["v"], dd["log_alpha"], dd["beta"],
                              h0=dd.get("h0"), cu_seqlens=dd.get("cu_seqlens"), scale=scale, check=True, **kw)
    torch.cuda.synchronize()
    for name, g in guards.items():
        g.assert_untouched(name)
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
