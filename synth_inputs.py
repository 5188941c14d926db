"""Seeded synthetic KDA inputs shared by tests, smoke and bench.

This module holds only the input recipe (random draws, normalisation, the
gate squashing functions and dtype casts).  None of the method's arithmetic
lives here, and neither the oracle nor the HIP package imports it: callers
generate tensors once and hand the very same values to both sides.

Recipe (per token and head): q, k ~ N(0,1) then L2-normalised over d_k;
v ~ N(0,1); beta = sigmoid(N(0,1)); log_alpha = -softplus(N(mu,1)) per key
channel; all math in fp32, cast to the requested dtype last (so bf16 q/k are
only approximately unit-norm; both sides take them as given).  Draw order is
fixed: q, k, v, beta-logit, gate-logit, h0.
"""
import numpy as np
import torch
import torch.nn.functional as F

# The five workload shapes of the build's baseline description.
CONFIGS = {
    "cfg0_tiny_fp32": dict(B=1, H=2, T=256, dk=64, dv=64, dtype="f32", mu=0.0, seed=0,
                           h0_std=0.0),
    "cfg1_prefill_bf16": dict(B=4, H=16, T=4096, dk=128, dv=128, dtype="bf16", mu=-2.0,
                              seed=0, h0_std=0.02),
    "cfg2_varlen_bf16": dict(N=8, len_lo=512, len_hi=8192, H=32, dk=128, dv=128,
                             dtype="bf16", mu=-2.0, seed=1, h0_std=0.0),
    "cfg3_long_bf16": dict(B=1, H=32, T=1048576, dk=128, dv=128, dtype="bf16", mu=-2.0,
                           seed=3, h0_std=0.0),
    "cfg4_decode_bf16": dict(N=256, H=32, dk=128, dv=128, dtype="bf16", mu=-2.0, seed=4,
                             state_std=0.02, steps=100),
}

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def torch_dtype(name):
    return _TORCH_DTYPE[name]


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def make_tokens(B, T, H, dk, dv, dtype="bf16", mu=-2.0, seed=0, device="cpu"):
    """Token tensors for a [B,T,H,*] problem.  Returns dict(q,k,v,log_alpha,beta)."""
    gen = _gen(seed, device)
    dt = _TORCH_DTYPE[dtype]

    def randn(*shape):
        return torch.randn(*shape, generator=gen, device=device, dtype=torch.float32)

    q = F.normalize(randn(B, T, H, dk), dim=-1)
    k = F.normalize(randn(B, T, H, dk), dim=-1)
    v = randn(B, T, H, dv)
    beta = torch.sigmoid(randn(B, T, H))
    log_alpha = -F.softplus(randn(B, T, H, dk) + mu)
    return dict(q=q.to(dt), k=k.to(dt), v=v.to(dt), log_alpha=log_alpha.to(dt),
                beta=beta.to(dt))


def make_raw_tokens(B, T, H, dk, dv, dtype="bf16", mu=-2.0, seed=0, device="cpu"):
    """Raw projections for the fused-prologue entry points, [B,T,H,*]: un-normalised q and k
    (N(0, 2^2)), v, gate logits N(mu, 1), beta logits N(0, 1), plus the decay-function constants
    a_scale [H] in [0.5, 2) and dt_bias [H,dk] ~ N(0, 0.5^2) in fp32.  No arithmetic of the method
    is applied here."""
    gen = _gen(seed + 104729, device)
    dt = _TORCH_DTYPE[dtype]

    def randn(*shape):
        return torch.randn(*shape, generator=gen, device=device, dtype=torch.float32)

    d = dict(q_raw=(2.0 * randn(B, T, H, dk)).to(dt), k_raw=(2.0 * randn(B, T, H, dk)).to(dt),
             v=randn(B, T, H, dv).to(dt), gate=(randn(B, T, H, dk) + mu).to(dt),
             beta_logit=randn(B, T, H).to(dt))
    d["a_scale"] = 0.5 + 1.5 * torch.rand(H, generator=gen, device=device, dtype=torch.float32)
    d["dt_bias"] = 0.5 * randn(H, dk)
    return d


def make_state(N, H, dk, dv, std, seed, device="cpu"):
    """fp32 state tensor [N,H,dk,dv] ~ N(0, std^2) (zeros if std == 0)."""
    if std == 0.0:
        return torch.zeros(N, H, dk, dv, dtype=torch.float32, device=device)
    gen = _gen(seed + 7919, device)
    return torch.randn(N, H, dk, dv, generator=gen, device=device,
                       dtype=torch.float32) * std


def make_prefill(B, T, H, dk, dv, dtype="bf16", mu=-2.0, seed=0, h0_std=0.0,
                 device="cpu"):
    """Fixed-length prefill problem.  Adds h0 (None when h0_std == 0)."""
    d = make_tokens(B, T, H, dk, dv, dtype, mu, seed, device)
    d["h0"] = make_state(B, H, dk, dv, h0_std, seed, device) if h0_std > 0 else None
    d["cu_seqlens"] = None
    return d


def varlen_lengths(N, lo, hi, seed):
    """Sequence lengths drawn uniformly from [lo, hi] (inclusive)."""
    return np.random.default_rng(seed).integers(lo, hi + 1, N).astype(np.int64)


def make_varlen(lengths, H, dk, dv, dtype="bf16", mu=-2.0, seed=1, h0_std=0.0,
                device="cpu"):
    """Packed variable-length problem: one token stream [1,sum(len),H,*]."""
    lengths = np.asarray(lengths, dtype=np.int64)
    total = int(lengths.sum())
    d = make_tokens(1, total, H, dk, dv, dtype, mu, seed, device)
    cu = np.zeros(len(lengths) + 1, dtype=np.int64)
    cu[1:] = np.cumsum(lengths)
    d["cu_seqlens"] = torch.from_numpy(cu.astype(np.int32)).to(device)
    d["h0"] = (make_state(len(lengths), H, dk, dv, h0_std, seed, device)
               if h0_std > 0 else None)
    return d


def make_long_on_device(T, H, dk, dv, dtype, mu, seed, device, block=65536):
    """[1,T,H,*] problem generated block by block on `device` to bound the fp32
    temporaries (block b uses seed + b).  Returns the same dict as make_tokens."""
    dt = _TORCH_DTYPE[dtype]
    out = dict(q=torch.empty(1, T, H, dk, dtype=dt, device=device),
               k=torch.empty(1, T, H, dk, dtype=dt, device=device),
               v=torch.empty(1, T, H, dv, dtype=dt, device=device),
               log_alpha=torch.empty(1, T, H, dk, dtype=dt, device=device),
               beta=torch.empty(1, T, H, dtype=dt, device=device))
    for b, t0 in enumerate(range(0, T, block)):
        t1 = min(t0 + block, T)
        part = make_tokens(1, t1 - t0, H, dk, dv, dtype, mu, seed + b, device)
        for name in out:
            out[name][:, t0:t1] = part[name]
        del part
    return out


def make_decode_tokens(N, H, dk, dv, dtype, mu, seed, step, device="cpu"):
    """Fresh tokens for decode step `step`: dict(q,k,v,log_alpha,beta) of [N,H,*]."""
    d = make_tokens(N, 1, H, dk, dv, dtype, mu, seed * 1000003 + step, device)
    return {name: t[:, 0].contiguous() for name, t in d.items()}


def to_np32(t):
    """Exact float32 numpy view of a tensor's values (bf16/fp32 -> float32)."""
    if t is None:
        return None
    return t.detach().to("cpu").to(torch.float32).numpy()
