"""fp64 CPU oracle for KDA -- TEST INFRASTRUCTURE, not product code.

Only tests, the smoke check and the CPU-baseline leg of the bench may import
this package.  It never imports the HIP package and shares no code with it.

`kda_forward` / `kda_step` / `kda_steps_pooled` call the plain C recurrence in ``kda_oracle.c``
(paper Section 3, Eq. (1)); `chunkwise_ref.kda_chunkwise` is a second, numpy
fp64 statement of the same function written from the chunkwise equations of
Section 3.1, used to pin the recurrence (chunk-size invariance).  `prologue` states the
input parameterisation of Section 4 (L2Norm, Sigmoid, the decay function) and `epilogue`
the output gate of the same section (head-wise RMSNorm times a sigmoid gate), in float64.
`kda_forward_scalar_gate` / `kda_steps_pooled_scalar_gate` are the scalar-gate special case of
Eq. (1) (Section 2.2, alpha_t = a_t I): the same recurrence on the decay repeated over the channels.
`kda_backward` is the reverse-mode derivative of that recurrence, token by token (the paper derives no
backward algorithm; the chain rule on Eq. (1) is the definition), pinned by finite differences of the
two forward statements.
"""
import numpy as _np

from . import epilogue, prologue  # noqa: F401
from .recurrence import build, kda_backward, kda_forward, kda_step, kda_steps_pooled, num_threads  # noqa: F401


def kda_forward_raw(q_raw, k_raw, v, gate, beta_logit, eps=1e-6, a_scale=None, dt_bias=None, **kw):
    """The recurrence behind the input parameterisation of Section 4: prologue.apply in float64,
    then kda_forward (which takes its inputs as float32: the one rounding, 6e-8 relative, that
    this adds is far below every tolerance it is compared under)."""
    q, k, log_alpha, beta = prologue.apply(q_raw, k_raw, gate, beta_logit, eps, a_scale, dt_bias)
    return kda_forward(q, k, v, log_alpha, beta, **kw)


def kda_forward_scalar_gate(q, k, v, log_alpha_head, beta, **kw):
    """Eq. (1) with one decay per (token, head), alpha_t = a_t I (Section 2.2): log_alpha_head is
    [B,T,H]; it is repeated over the dk channels and handed to the per-channel recurrence."""
    la = _np.asarray(log_alpha_head)
    full = _np.ascontiguousarray(_np.broadcast_to(la[..., None], _np.asarray(q).shape))
    return kda_forward(q, k, v, full, beta, **kw)


def kda_steps_pooled_scalar_gate(q, k, v, log_alpha_head, beta, S_pool, state_indices=None, **kw):
    """kda_steps_pooled with one decay per (token, head): log_alpha_head is [N,Tq,H]."""
    la = _np.asarray(log_alpha_head)
    full = _np.ascontiguousarray(_np.broadcast_to(la[..., None], _np.asarray(q).shape))
    return kda_steps_pooled(q, k, v, full, beta, S_pool, state_indices, **kw)
