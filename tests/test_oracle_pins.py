"""Pins for the fp64 oracle: closed forms, reductions, invariants, brute force.

The paper prints no worked numeric example of KDA, so every pin here is
something the paper or the mathematics fixes independently of the oracle's
own code.  Each test names the passage it rests on.
"""
import numpy as np
import pytest

import oracle
from oracle.chunkwise_ref import kda_chunkwise


def _inputs(rng, B, T, H, dk, dv, mu=0.0, unit_k=True):
    q = rng.standard_normal((B, T, H, dk))
    k = rng.standard_normal((B, T, H, dk))
    if unit_k:
        q /= np.linalg.norm(q, axis=-1, keepdims=True)
        k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = rng.standard_normal((B, T, H, dv))
    beta = 1.0 / (1.0 + np.exp(-rng.standard_normal((B, T, H))))
    g = -np.log1p(np.exp(rng.standard_normal((B, T, H, dk)) + mu))
    # the oracle reads float32 values: round once here so both sides see the same
    f = lambda a: a.astype(np.float32)
    return f(q), f(k), f(v), f(g), f(beta)


def test_bruteforce_unrolled_product():
    """Section 3.1, chunk expansion S^r = P^r S^0 + H^r with explicit d_k x d_k
    transition matrices (I - beta k k^T) Diag(alpha), T <= 8."""
    rng = np.random.default_rng(10)
    for T, dk, dv in [(1, 2, 3), (5, 3, 2), (8, 4, 4)]:
        q, k, v, g, b = _inputs(rng, 1, T, 1, dk, dv, unit_k=False)
        S0 = rng.standard_normal((1, 1, dk, dv))
        o, hT = oracle.kda_forward(q, k, v, g, b, h0=S0)
        kk, vv, gg, bb, qq = (x[0, :, 0].astype(np.float64) for x in (k, v, g, b, q))
        trans = [(np.eye(dk) - bb[t] * np.outer(kk[t], kk[t])) @ np.diag(np.exp(gg[t]))
                 for t in range(T)]
        for r in range(1, T + 1):
            P = np.eye(dk)
            for i in range(r):                  # P^r = T_r ... T_1
                P = trans[i] @ P
            Hr = np.zeros((dk, dv))
            for i in range(r):                  # token i+1 (1-based) write, then T_{i+2..r}
                term = bb[i] * np.outer(kk[i], vv[i])
                for j in range(i + 1, r):
                    term = trans[j] @ term
                Hr += term
            S_r = P @ S0[0, 0] + Hr
            np.testing.assert_allclose(o[0, r - 1, 0], S_r.T @ qq[r - 1], rtol=0, atol=1e-13)
        np.testing.assert_allclose(hT[0, 0], S_r, rtol=0, atol=1e-13)


def test_reduces_to_deltanet_when_alpha_is_one():
    """Section 2.2 (DeltaNet): S_t = S_{t-1} - beta_t k_t (S_{t-1}^T k_t - v_t)^T."""
    rng = np.random.default_rng(11)
    B, T, H, dk, dv = 2, 37, 2, 8, 5
    q, k, v, g, b = _inputs(rng, B, T, H, dk, dv)
    g[:] = 0.0
    o, hT = oracle.kda_forward(q, k, v, g, b)
    for bi in range(B):
        for h in range(H):
            S = np.zeros((dk, dv))
            for t in range(T):
                kt, vt = k[bi, t, h].astype(np.float64), v[bi, t, h].astype(np.float64)
                grad = np.outer(kt, S.T @ kt - vt)     # gradient of 1/2 |S^T k - v|^2
                S = S - float(b[bi, t, h]) * grad
                np.testing.assert_allclose(o[bi, t, h], S.T @ q[bi, t, h].astype(np.float64),
                                           rtol=0, atol=1e-13)
            np.testing.assert_allclose(hT[bi, h], S, rtol=0, atol=1e-13)


def test_reduces_to_gdn_when_alpha_is_channel_constant():
    """Section 2.2 (Gated DeltaNet): S_t = a_t (I - beta k k^T) S_{t-1} + beta k v^T."""
    rng = np.random.default_rng(12)
    B, T, H, dk, dv = 1, 29, 3, 6, 7
    q, k, v, g, b = _inputs(rng, B, T, H, dk, dv)
    g[:] = g[..., :1]                                   # same log-decay on every channel
    h0 = rng.standard_normal((B, H, dk, dv))
    o, hT = oracle.kda_forward(q, k, v, g, b, h0=h0)
    for h in range(H):
        S = h0[0, h].copy()
        for t in range(T):
            kt, vt = k[0, t, h].astype(np.float64), v[0, t, h].astype(np.float64)
            a = np.exp(np.float64(g[0, t, h, 0]))
            bt = np.float64(b[0, t, h])
            S = a * (np.eye(dk) - bt * np.outer(kt, kt)) @ S + bt * np.outer(kt, vt)
            np.testing.assert_allclose(o[0, t, h], S.T @ q[0, t, h].astype(np.float64),
                                       rtol=0, atol=1e-12)
        np.testing.assert_allclose(hT[0, h], S, rtol=0, atol=1e-12)


def test_scalar_gate_entry_equals_the_scalar_recurrence_written_out():
    """kda_forward_scalar_gate / kda_steps_pooled_scalar_gate against Section 2.2's recurrence with
    a scalar a_t, written out here with explicit matrices."""
    rng = np.random.default_rng(121)
    B, T, H, dk, dv = 2, 17, 2, 5, 4
    q, k, v, g, b = _inputs(rng, B, T, H, dk, dv)
    gh = np.ascontiguousarray(g[..., 0])                  # [B,T,H]
    h0 = rng.standard_normal((B, H, dk, dv))
    o, hT = oracle.kda_forward_scalar_gate(q, k, v, gh, b, h0=h0, scale=0.7)
    o_p, pool = oracle.kda_steps_pooled_scalar_gate(q[:, :6], k[:, :6], v[:, :6], gh[:, :6], b[:, :6], h0, scale=0.7)
    for bi in range(B):
        for h in range(H):
            S = h0[bi, h].copy()
            for t in range(T):
                kt, vt = k[bi, t, h].astype(np.float64), v[bi, t, h].astype(np.float64)
                a, bt = np.exp(np.float64(gh[bi, t, h])), np.float64(b[bi, t, h])
                S = a * (np.eye(dk) - bt * np.outer(kt, kt)) @ S + bt * np.outer(kt, vt)
                ot = 0.7 * (S.T @ q[bi, t, h].astype(np.float64))
                np.testing.assert_allclose(o[bi, t, h], ot, rtol=0, atol=1e-12)
                if t < 6:
                    np.testing.assert_allclose(o_p[bi, t, h], ot, rtol=0, atol=1e-12)
                if t == 5:
                    np.testing.assert_allclose(pool[bi, h], S, rtol=0, atol=1e-12)
            np.testing.assert_allclose(hT[bi, h], S, rtol=0, atol=1e-12)


def test_beta_zero_is_pure_decay_of_h0():
    """Eq. (1) with beta = 0: S_t = Diag(prod alpha) h0, o_t = (Gamma_t . q_t)^T h0."""
    rng = np.random.default_rng(13)
    B, T, H, dk, dv = 1, 50, 2, 5, 4
    q, k, v, g, b = _inputs(rng, B, T, H, dk, dv)
    b[:] = 0.0
    h0 = rng.standard_normal((B, H, dk, dv))
    o, hT = oracle.kda_forward(q, k, v, g, b, h0=h0)
    G = np.cumsum(g.astype(np.float64), axis=1)
    for h in range(H):
        np.testing.assert_allclose(hT[0, h], np.exp(G[0, -1, h])[:, None] * h0[0, h],
                                   rtol=1e-13, atol=1e-300)
        for t in range(T):
            want = (np.exp(G[0, t, h]) * q[0, t, h].astype(np.float64)) @ h0[0, h]
            np.testing.assert_allclose(o[0, t, h], want, rtol=0, atol=1e-13)


def test_whole_sequence_closed_form():
    """Section 6.1, table of parallel forms, KDA row (with beta restored and the
    strict mask read for the garbled symbol), h0 = 0:
    O = Tril(A_qk) (I + StrictTril(Diag(beta) A_kk))^-1 Diag(beta) V with
    A_xk[r,i] = sum_d x_r k_i exp(G_r - G_i), solved with numpy.linalg.solve."""
    rng = np.random.default_rng(14)
    T, dk, dv = 48, 6, 5
    q, k, v, g, b = _inputs(rng, 1, T, 1, dk, dv)
    o, _ = oracle.kda_forward(q, k, v, g, b)
    Q, K, V, bb = (x[0, :, 0].astype(np.float64) for x in (q, k, v, b))
    G = np.cumsum(g[0, :, 0].astype(np.float64), axis=0)
    Aqk = np.zeros((T, T))
    Akk = np.zeros((T, T))
    for r in range(T):
        for i in range(r + 1):
            dec = np.exp(G[r] - G[i])
            Aqk[r, i] = np.sum(Q[r] * K[i] * dec)
            Akk[r, i] = np.sum(K[r] * K[i] * dec)
    L = np.tril(bb[:, None] * Akk, -1)
    X = np.linalg.solve(np.eye(T) + L, bb[:, None] * V)
    np.testing.assert_allclose(o[0, :, 0], np.tril(Aqk) @ X, rtol=0, atol=1e-12)


def test_one_step_invariant_unit_keys():
    """Delta-rule property (Section 2.2): for |k_t| = 1,
    S_t^T k_t = (1 - beta_t)(Diag(alpha_t) S_{t-1})^T k_t + beta_t v_t; with beta_t = 1
    the memory returns v_t exactly when probed with k_t."""
    rng = np.random.default_rng(15)
    N, H, dk, dv = 3, 2, 4, 6
    # unit keys that are exact in float32: signed, scaled one/two-hot patterns
    k = np.zeros((N, H, dk), np.float32)
    for n in range(N):
        for h in range(H):
            if (n + h) % 2 == 0:
                k[n, h, (n + h) % dk] = -1.0
            else:
                k[n, h, :] = 0.5 * np.where(rng.random(dk) < 0.5, -1.0, 1.0)  # |k|=1 for dk=4
    q = k.copy()
    v = rng.standard_normal((N, H, dv)).astype(np.float32)
    g = (-np.log1p(np.exp(rng.standard_normal((N, H, dk))))).astype(np.float32)
    S = rng.standard_normal((N, H, dk, dv))
    for beta_val in (1.0, 0.25):
        b = np.full((N, H), beta_val, np.float32)
        o, S1 = oracle.kda_step(q, k, v, g, b, S)
        dec = np.exp(g.astype(np.float64))[..., None] * S
        pred = np.einsum("nhkv,nhk->nhv", dec, k.astype(np.float64))
        want = (1.0 - beta_val) * pred + beta_val * v.astype(np.float64)
        np.testing.assert_allclose(o, want, rtol=0, atol=1e-14)
        np.testing.assert_allclose(np.einsum("nhkv,nhk->nhv", S1, k.astype(np.float64)),
                                   want, rtol=0, atol=1e-14)
        if beta_val == 1.0:
            np.testing.assert_allclose(o, v.astype(np.float64), rtol=0, atol=1e-14)


def test_one_hot_keys_give_diagonal_transitions():
    """With k_t = e_pi(t) every transition of Eq. (1) is diagonal, so state row j
    follows row_j <- alpha_t[j] (1 - beta_t [j=pi(t)]) row_j + beta_t [j=pi(t)] v_t."""
    rng = np.random.default_rng(16)
    T, dk, dv = 6, 6, 3
    perm = rng.permutation(dk)[:T]
    k = np.zeros((1, T, 1, dk), np.float32)
    k[0, np.arange(T), 0, perm] = 1.0
    q, _, v, g, b = _inputs(rng, 1, T, 1, dk, dv)
    h0 = rng.standard_normal((1, 1, dk, dv))
    o, hT = oracle.kda_forward(q, k, v, g, b, h0=h0)
    rows = h0[0, 0].copy()
    for t in range(T):
        a = np.exp(g[0, t, 0].astype(np.float64))
        for j in range(dk):
            hit = 1.0 if perm[t] == j else 0.0
            rows[j] = a[j] * (1.0 - float(b[0, t, 0]) * hit) * rows[j] \
                + float(b[0, t, 0]) * hit * v[0, t, 0].astype(np.float64)
        np.testing.assert_allclose(o[0, t, 0], rows.T @ q[0, t, 0].astype(np.float64),
                                   rtol=0, atol=1e-14)
    np.testing.assert_allclose(hT[0, 0], rows, rtol=0, atol=1e-14)


@pytest.mark.parametrize("C", [1, 7, 16, 64, 100])
def test_chunk_size_invariance(C):
    """Section 3.1 / Appendix B: the chunkwise form (WY + UT transform + chunk state
    update + inter/intra output) equals the recurrence for every chunk size,
    including chunks that do not divide T."""
    rng = np.random.default_rng(17)
    B, T, H, dk, dv = 1, 100, 2, 8, 6
    q, k, v, g, b = _inputs(rng, B, T, H, dk, dv)
    h0 = 0.3 * rng.standard_normal((B, H, dk, dv))
    o, hT = oracle.kda_forward(q, k, v, g, b, h0=h0, scale=0.5)
    o2, hT2 = kda_chunkwise(q, k, v, g, b, h0=h0, C=C, scale=0.5)
    np.testing.assert_allclose(o, o2, rtol=0, atol=1e-12)
    np.testing.assert_allclose(hT, hT2, rtol=0, atol=1e-12)


def test_split_and_resume():
    """Section 2.1: the state after a prefix is the initial state of the rest."""
    rng = np.random.default_rng(18)
    B, T, H, dk, dv = 2, 61, 2, 8, 8
    q, k, v, g, b = _inputs(rng, B, T, H, dk, dv)
    o, hT = oracle.kda_forward(q, k, v, g, b)
    s = 23
    o1, h1 = oracle.kda_forward(q[:, :s], k[:, :s], v[:, :s], g[:, :s], b[:, :s])
    o2, h2 = oracle.kda_forward(q[:, s:], k[:, s:], v[:, s:], g[:, s:], b[:, s:], h0=h1)
    np.testing.assert_array_equal(np.concatenate([o1, o2], axis=1), o)
    np.testing.assert_array_equal(h2, hT)


def test_packed_equals_unpacked_and_empty_sequences():
    """Packed batches: each sequence is an independent run of Eq. (1) from its own
    h0; a zero-length sequence returns h0 unchanged."""
    rng = np.random.default_rng(19)
    H, dk, dv = 2, 4, 5
    lens = [5, 0, 9, 1]
    cu = np.concatenate([[0], np.cumsum(lens)])
    T = int(cu[-1])
    q, k, v, g, b = _inputs(rng, 1, T, H, dk, dv)
    h0 = rng.standard_normal((len(lens), H, dk, dv))
    o, hT = oracle.kda_forward(q, k, v, g, b, h0=h0, cu_seqlens=cu)
    for n, (s, e) in enumerate(zip(cu[:-1], cu[1:])):
        if e == s:
            np.testing.assert_array_equal(hT[n], h0[n])
            continue
        on, hn = oracle.kda_forward(q[:, s:e], k[:, s:e], v[:, s:e], g[:, s:e], b[:, s:e],
                                    h0=h0[n:n + 1])
        np.testing.assert_array_equal(o[:, s:e], on)
        np.testing.assert_array_equal(hT[n], hn[0])


def test_scale_is_linear_and_heads_are_independent():
    """o is linear in the query scale (App. C folds d_k^-1/2 into q); heads and
    batch rows never interact (Section 4: 'for each head h')."""
    rng = np.random.default_rng(20)
    B, T, H, dk, dv = 2, 20, 3, 4, 4
    q, k, v, g, b = _inputs(rng, B, T, H, dk, dv)
    o1, h1 = oracle.kda_forward(q, k, v, g, b)
    o2, h2 = oracle.kda_forward(q, k, v, g, b, scale=dk ** -0.5)
    np.testing.assert_allclose(o2, o1 * dk ** -0.5, rtol=1e-15, atol=0)
    np.testing.assert_array_equal(h1, h2)
    perm = [2, 0, 1]
    o3, h3 = oracle.kda_forward(q[:, :, perm], k[:, :, perm], v[:, :, perm], g[:, :, perm],
                                b[:, :, perm])
    np.testing.assert_array_equal(o3, o1[:, :, perm])
    np.testing.assert_array_equal(h3, h1[:, perm])


def test_suffix_oracle_contraction_bound():
    """|I - beta k k^T|_2 <= 1 for |k| <= 1, beta in [0,1], so the influence of the
    state at time s on the state at time T is at most exp(max_d sum_{t>s} log alpha).
    The recurrence run on a suffix from a zero state must match the full run to
    within that bound times the norm of the state it ignored."""
    rng = np.random.default_rng(21)
    B, T, H, dk, dv = 1, 400, 1, 8, 8
    q, k, v, g, b = _inputs(rng, B, T, H, dk, dv, mu=-4.0)
    _, hT = oracle.kda_forward(q, k, v, g, b)
    s = 250
    _, h_s = oracle.kda_forward(q[:, :s], k[:, :s], v[:, :s], g[:, :s], b[:, :s])
    _, h_suffix = oracle.kda_forward(q[:, s:], k[:, s:], v[:, s:], g[:, s:], b[:, s:])
    bound = np.exp(np.max(np.sum(g[0, s:, 0].astype(np.float64), axis=0)))
    diff = np.linalg.norm(hT[0, 0] - h_suffix[0, 0], 2)
    assert diff <= bound * np.linalg.norm(h_s[0, 0], 2) * (1 + 1e-9) + 1e-15
    assert diff > 0  # the bound is not vacuous here


def test_planted_mistakes_are_caught():
    """Sanity of the pins themselves: plausible wrong readings of Eq. (1) (decay after
    the correction, decayed write, output from the old state) disagree with the
    closed-form pin by far more than rounding."""
    rng = np.random.default_rng(22)
    T, dk, dv = 12, 4, 3
    q, k, v, g, b = _inputs(rng, 1, T, 1, dk, dv)
    o, _ = oracle.kda_forward(q, k, v, g, b)
    Q, K, V, bb, gg = (x[0, :, 0].astype(np.float64) for x in (q, k, v, b, g))

    def run(variant):
        S = np.zeros((dk, dv))
        out = np.zeros((T, dv))
        for t in range(T):
            a = np.exp(gg[t])[:, None]
            if variant == "decay_after":
                S = S + bb[t] * np.outer(K[t], V[t] - S.T @ K[t])
                S = a * S
                out[t] = S.T @ Q[t]
            elif variant == "decayed_write":
                S = a * (S + bb[t] * np.outer(K[t], V[t] - (a * S).T @ K[t]))
                out[t] = S.T @ Q[t]
            elif variant == "old_state_output":
                out[t] = S.T @ Q[t]
                S = a * S
                S = S + bb[t] * np.outer(K[t], V[t] - S.T @ K[t])
        return out

    for variant in ("decay_after", "decayed_write", "old_state_output"):
        assert np.max(np.abs(run(variant) - o[0, :, 0])) > 1e-3


def test_pooled_multi_token_decode_is_successive_single_steps_on_the_named_states():
    """Section 6.3: a multi-token decode over a state pool is Eq. (1) applied token by token to
    the state each sequence names; states nobody names stay as they were, skipped sequences
    produce no output."""
    rng = np.random.default_rng(5)
    N, Tq, H, dk, dv, P = 4, 3, 2, 8, 6, 7
    q = rng.standard_normal((N, Tq, H, dk)); k = rng.standard_normal((N, Tq, H, dk))
    k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = rng.standard_normal((N, Tq, H, dv))
    g = -np.log1p(np.exp(rng.standard_normal((N, Tq, H, dk))))
    b = 1.0 / (1.0 + np.exp(-rng.standard_normal((N, Tq, H))))
    pool = rng.standard_normal((P, H, dk, dv))
    idx = np.array([5, -1, 0, 3])
    f = lambda x: x.astype(np.float32)
    o, new = oracle.kda_steps_pooled(f(q), f(k), f(v), f(g), f(b), pool, idx, scale=0.5)
    # by hand: explicit transition matrices of Eq. (1), token by token
    for n in range(N):
        if idx[n] < 0:
            assert np.isnan(o[n]).all()
            continue
        for h in range(H):
            S = pool[idx[n], h].copy()
            for t in range(Tq):
                kk = f(k)[n, t, h].astype(np.float64); a = np.exp(f(g)[n, t, h].astype(np.float64))
                bb = float(f(b)[n, t, h])
                S = (np.eye(dk) - bb * np.outer(kk, kk)) @ (a[:, None] * S) + bb * np.outer(kk, f(v)[n, t, h].astype(np.float64))
                np.testing.assert_allclose(o[n, t, h], 0.5 * S.T @ f(q)[n, t, h].astype(np.float64), rtol=1e-11, atol=1e-12)
            np.testing.assert_allclose(new[idx[n], h], S, rtol=1e-11, atol=1e-12)
    untouched = [p_ for p_ in range(P) if p_ not in idx]
    assert np.array_equal(new[untouched], pool[untouched])


def test_prologue_closed_forms():
    """Input parameterisation (Section 4): each piece against a formula written differently."""
    from oracle import prologue as pro
    rng = np.random.default_rng(9)
    x = rng.standard_normal((3, 5, 2, 16)) * 3
    y = pro.l2norm(x, 0.0)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(pro.l2norm(7.5 * x, 0.0), y, rtol=1e-13)           # scale invariant
    np.testing.assert_allclose(pro.l2norm(x, 0.25), x / np.sqrt((x ** 2).sum(-1, keepdims=True) + 0.25), rtol=1e-14)
    z = rng.standard_normal(1000) * 6
    assert pro.sigmoid(0.0) == 0.5
    np.testing.assert_allclose(pro.sigmoid(z) + pro.sigmoid(-z), 1.0, rtol=1e-14)
    np.testing.assert_allclose(pro.sigmoid(z), np.exp(z) / (1 + np.exp(z)), rtol=1e-12)
    np.testing.assert_allclose(pro.softplus(z) - pro.softplus(-z), z, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(pro.softplus(0.0), np.log(2.0), rtol=1e-15)
    np.testing.assert_allclose(pro.softplus(50.0), 50.0, rtol=1e-15)
    np.testing.assert_allclose(pro.softplus(-40.0), np.exp(-40.0), rtol=1e-12)
    # alpha = sigmoid(-(gate + bias)) ** a_scale, per head and channel
    gate = rng.standard_normal((2, 7, 3, 16)) * 2
    a = np.array([0.5, 1.0, 3.0]); bias = rng.standard_normal((3, 16))
    la = pro.log_alpha_from_gate(gate, a, bias)
    np.testing.assert_allclose(np.exp(la), pro.sigmoid(-(gate + bias)) ** a[:, None], rtol=1e-12)
    assert (la < 0).all()
    # the baseline workloads draw log alpha = -softplus(logit): a_scale = 1, bias = 0
    np.testing.assert_allclose(pro.log_alpha_from_gate(gate), -np.log1p(np.exp(gate)), rtol=1e-12)


def test_forward_raw_composes_prologue_and_recurrence():
    rng = np.random.default_rng(10)
    B, T, H, dk, dv = 1, 9, 2, 8, 4
    qr, kr = rng.standard_normal((2, B, T, H, dk)) * 2
    v = rng.standard_normal((B, T, H, dv)); gate = rng.standard_normal((B, T, H, dk)); bl = rng.standard_normal((B, T, H))
    o, hT = oracle.kda_forward_raw(qr, kr, v, gate, bl, eps=0.0)
    # by hand, with explicit transition matrices of Eq. (1)
    for h in range(H):
        S = np.zeros((dk, dv))
        for t in range(T):
            kk = kr[0, t, h] / np.linalg.norm(kr[0, t, h]); qq = qr[0, t, h] / np.linalg.norm(qr[0, t, h])
            al = 1.0 / (1.0 + np.exp(gate[0, t, h])); be = 1.0 / (1.0 + np.exp(-bl[0, t, h]))
            S = (np.eye(dk) - be * np.outer(kk, kk)) @ (al[:, None] * S) + be * np.outer(kk, v[0, t, h])
            np.testing.assert_allclose(o[0, t, h], S.T @ qq, rtol=2e-6, atol=2e-7)
        np.testing.assert_allclose(hT[0, h], S, rtol=2e-6, atol=2e-7)


def test_epilogue_closed_forms():
    """Output gate (Section 4): head-wise RMSNorm times Sigmoid(gate), against other formulas."""
    from oracle import epilogue as epi
    rng = np.random.default_rng(12)
    o = rng.standard_normal((2, 5, 3, 16)) * 4
    y = epi.rmsnorm(o, None, 0.0)
    np.testing.assert_allclose(np.mean(y * y, axis=-1), 1.0, rtol=1e-13)          # unit mean square
    np.testing.assert_allclose(epi.rmsnorm(-3.0 * o, None, 0.0), -y, rtol=1e-13)  # scale invariant, odd
    np.testing.assert_allclose(y, o * np.sqrt(16) / np.linalg.norm(o, axis=-1, keepdims=True), rtol=1e-13)
    w = rng.standard_normal(16)
    np.testing.assert_allclose(epi.rmsnorm(o, w, 0.5), o / np.sqrt((o ** 2).mean(-1, keepdims=True) + 0.5) * w,
                               rtol=1e-14)
    g = rng.standard_normal(o.shape) * 3
    out = epi.apply(o, g, w, 0.5)
    np.testing.assert_allclose(out, epi.rmsnorm(o, w, 0.5) * np.exp(g) / (1 + np.exp(g)), rtol=1e-12)
    np.testing.assert_allclose(epi.apply(o, np.zeros_like(o), w, 0.5), 0.5 * epi.rmsnorm(o, w, 0.5), rtol=1e-15)
    big = epi.apply(o, np.full_like(o, 40.0), None, 0.0)
    np.testing.assert_allclose(big, y, rtol=1e-12)                                  # open gate
