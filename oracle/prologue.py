"""fp64 statement of the input parameterisation that precedes KDA -- TEST INFRASTRUCTURE.

Section 4 ("Neural Parameterization") feeds the recurrence with
    q, k = L2Norm(.)            over the key head dimension,
    beta = Sigmoid(.)           per head,
    alpha = f(.)                per key channel, f "similar to GDN and Mamba".
The paper does not print f.  The reading taken here is the one of those two models, which is
also how the baseline workloads draw their decays:
    log alpha = -a_scale[h] * softplus(gate + dt_bias[h, c]),      softplus(x) = log(1 + e^x),
with a_scale = 1 and dt_bias = 0 giving log alpha = -softplus(gate).  The projections, the short
convolution and Swish need weights and stay outside.  L2Norm is x / sqrt(sum x^2 + eps).

Plain numpy, float64 throughout; nothing here is shared with the HIP path.
"""
import numpy as np


def l2norm(x, eps):
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt(np.sum(x * x, axis=-1, keepdims=True) + eps)


def sigmoid(x):
    x = np.asarray(x, dtype=np.float64)
    return 1.0 / (1.0 + np.exp(-x))


def softplus(x):
    x = np.asarray(x, dtype=np.float64)
    return np.maximum(x, 0.0) + np.log1p(np.exp(-np.abs(x)))


def log_alpha_from_gate(gate, a_scale=None, dt_bias=None):
    """gate [..., H, dk]; a_scale [H] or None (= 1); dt_bias [H, dk] or None (= 0)."""
    x = np.asarray(gate, dtype=np.float64)
    if dt_bias is not None:
        x = x + np.asarray(dt_bias, dtype=np.float64)
    s = softplus(x)
    if a_scale is not None:
        s = s * np.asarray(a_scale, dtype=np.float64)[:, None]
    return -s


def apply(q_raw, k_raw, gate, beta_logit, eps=1e-6, a_scale=None, dt_bias=None):
    """Raw projections -> (q, k, log_alpha, beta) as the recurrence takes them, float64."""
    return (l2norm(q_raw, eps), l2norm(k_raw, eps), log_alpha_from_gate(gate, a_scale, dt_bias),
            sigmoid(beta_logit))
