"""Chunkwise KDA in numpy fp64 -- TEST INFRASTRUCTURE, not product code.

A second statement of the KDA forward pass, written from the chunkwise
equations of the paper's Section 3.1 (WY representation, UT transform, chunk
state update and the inter/intra-chunk output), one head at a time.  Its only
job is to pin the per-token recurrence oracle: the paper claims the chunkwise
form equals the recurrence for every chunk size, so the two must agree to
fp64 rounding for any C, including chunks that do not divide T.

Reading of the decay notation used here: gamma^{i->r} is the product of
alpha over tokens i+1..r (exclusive of i), i.e. exp(G^r - G^i) with G the
inclusive cumulative sum of log alpha inside the chunk.  This is the reading
under which the propositions of Appendix B hold (gamma^{r->r} = 1).
"""
import numpy as np


def kda_chunkwise_head(q, k, v, g, beta, S0, C, scale=1.0):
    """One (sequence, head): q,k,g [T,dk], v [T,dv], beta [T], S0 [dk,dv]."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64)
    g = np.asarray(g, np.float64)
    beta = np.asarray(beta, np.float64)
    S = np.array(S0, np.float64, copy=True)
    T, dv = v.shape
    o = np.zeros((T, dv))
    for c0 in range(0, T, C):
        c1 = min(c0 + C, T)
        n = c1 - c0
        Q, K, V, b = q[c0:c1], k[c0:c1], v[c0:c1], beta[c0:c1]
        G = np.cumsum(g[c0:c1], axis=0)                  # [n,dk], inclusive
        # pairwise decay exp(G^r - G^i); only r >= i is ever used, where it is <= 1
        D = np.exp(np.minimum(G[:, None, :] - G[None, :, :], 0.0))      # [r,i,dk]
        Akk = np.einsum("rd,id,rid->ri", K, K, D)
        Aqk = np.einsum("rd,id,rid->ri", Q, K, D)
        L = np.tril(b[:, None] * Akk, -1)                # StrictTril(Diag(beta) ...)
        M = np.linalg.solve(np.eye(n) + L, np.diag(b))   # (I + L)^-1 Diag(beta)
        W = M @ (np.exp(G) * K)                          # M (Gamma . K)
        U = M @ V
        Vnew = U - W @ S                                 # "pseudo"-value term
        o[c0:c1] = scale * ((np.exp(G) * Q) @ S + np.tril(Aqk) @ Vnew)
        Kdec = np.exp(G[-1][None, :] - G) * K            # Gamma^{i->C} . K
        S = np.exp(G[-1])[:, None] * S + Kdec.T @ Vnew
    return o, S


def kda_chunkwise(q, k, v, log_alpha, beta, h0=None, C=64, scale=1.0):
    """Batched wrapper: q,k,log_alpha [B,T,H,dk], v [B,T,H,dv], beta [B,T,H]."""
    q = np.asarray(q)
    B, T, H, dk = q.shape
    dv = np.asarray(v).shape[-1]
    o = np.zeros((B, T, H, dv))
    hT = np.zeros((B, H, dk, dv))
    for b in range(B):
        for h in range(H):
            S0 = np.zeros((dk, dv)) if h0 is None else np.asarray(h0)[b, h]
            o[b, :, h], hT[b, h] = kda_chunkwise_head(
                np.asarray(q)[b, :, h], np.asarray(k)[b, :, h], np.asarray(v)[b, :, h],
                np.asarray(log_alpha)[b, :, h], np.asarray(beta)[b, :, h], S0, C, scale)
    return o, hT
