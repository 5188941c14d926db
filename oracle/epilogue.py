"""fp64 statement of the output gate that follows KDA -- TEST INFRASTRUCTURE.

Section 4 ("Neural Parameterization"): before the output projection the layer applies a
head-wise RMSNorm to the KDA output and multiplies by a sigmoid gate,
    y = Sigmoid(g) * RMSNorm(o),      RMSNorm(o) = o / sqrt(mean_j o_j^2 + eps) * w,
where the mean runs over the d_v values of one (token, head).  The paper gives neither eps nor
the shape of the learned weight; the reading taken here is one weight vector of length d_v shared
by all heads (None = ones) and eps as a parameter.  The gate's own low-rank projection and the
output projection need weights and stay outside.

Plain numpy, float64 throughout; nothing here is shared with the HIP path.
"""
import numpy as np


def rmsnorm(o, weight=None, eps=1e-6):
    o = np.asarray(o, dtype=np.float64)
    y = o / np.sqrt(np.mean(o * o, axis=-1, keepdims=True) + eps)
    return y if weight is None else y * np.asarray(weight, dtype=np.float64)


def apply(o, gate, weight=None, eps=1e-6):
    """o, gate: [..., H, dv]; weight: [dv] or None.  Returns Sigmoid(gate) * RMSNorm(o)."""
    g = np.asarray(gate, dtype=np.float64)
    return rmsnorm(o, weight, eps) / (1.0 + np.exp(-g))
