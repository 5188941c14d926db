"""Pins for the backward oracle (reverse-mode derivative of Section 3, Eq. (1)).

The paper derives no backward pass, so what fixes the gradients is the forward function itself:
finite differences of the two independent forward statements (the chunkwise numpy form of
Section 3.1 in float64, and the C recurrence), closed forms for one token, and identities that hold
because the output is linear in some of the inputs.  A dropped term, a wrong sign, a transposed
operand or an off-by-one in the order of decay and update changes at least one of them.
"""
import numpy as np
import pytest

import oracle
from oracle.chunkwise_ref import kda_chunkwise


def _inputs(rng, B, T, H, dk, dv, mu=0.0):
    q = rng.standard_normal((B, T, H, dk))
    k = rng.standard_normal((B, T, H, dk)) / np.sqrt(dk)
    v = rng.standard_normal((B, T, H, dv))
    beta = 1.0 / (1.0 + np.exp(-rng.standard_normal((B, T, H))))
    g = -np.log1p(np.exp(rng.standard_normal((B, T, H, dk)) + mu))
    f = lambda a: a.astype(np.float32)
    return f(q), f(k), f(v), f(g), f(beta)


NAMES = ["dq", "dk", "dv", "dlog_alpha", "dbeta", "dh0"]


def test_every_gradient_entry_against_central_differences_of_the_chunkwise_form():
    """Element by element, every input: (L(x + h e) - L(x - h e)) / 2h with the float64 chunkwise
    forward (Section 3.1; chunk 4 does not divide T = 10), h = 1e-6; d_k != d_v so that a transposed
    state shows; scale != 1; final-state gradient and initial state present."""
    rng = np.random.default_rng(101)
    B, T, H, dk, dv = 1, 10, 2, 3, 5
    q, k, v, g, b = _inputs(rng, B, T, H, dk, dv)
    h0 = rng.standard_normal((B, H, dk, dv)).astype(np.float32)
    do = rng.standard_normal((B, T, H, dv))
    dhT = rng.standard_normal((B, H, dk, dv))
    scale = 0.7
    grads = oracle.kda_backward(q, k, v, g, b, do, dhT=dhT, h0=h0, scale=scale)

    base = [x.astype(np.float64) for x in (q, k, v, g, b, h0)]

    def loss(args):
        o, hT = kda_chunkwise(args[0], args[1], args[2], args[3], args[4], h0=args[5], C=4, scale=scale)
        return float((o * do).sum() + (hT * dhT).sum())

    h = 1e-6
    for which, name in enumerate(NAMES):
        num = np.zeros_like(base[which])
        it = np.nditer(base[which], flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            plus = [a.copy() for a in base]
            minus = [a.copy() for a in base]
            plus[which][idx] += h
            minus[which][idx] -= h
            num[idx] = (loss(plus) - loss(minus)) / (2 * h)
        err = np.abs(grads[name] - num).max() / max(np.abs(num).max(), 1e-30)
        assert err < 2e-7, (name, err)


def test_directional_derivatives_of_the_c_recurrence_with_exact_perturbations():
    """The C forward reads float32 inputs, so the perturbation is chosen exactly representable:
    inputs rounded to 2^-7, step 2^-12 along a random +-1 direction.  The central difference of a
    smooth function is off by O(step^2)."""
    rng = np.random.default_rng(102)
    B, T, H, dk, dv = 2, 70, 2, 8, 6
    arrs = [np.round(x.astype(np.float64) * 128) / 128 for x in _inputs(rng, B, T, H, dk, dv)]
    arrs[3] = -np.abs(arrs[3]) - 1.0 / 128           # log alpha stays negative
    h0 = np.round(rng.standard_normal((B, H, dk, dv)) * 128) / 128
    do = rng.standard_normal((B, T, H, dv))
    dhT = rng.standard_normal((B, H, dk, dv))
    grads = oracle.kda_backward(*arrs, do, dhT=dhT, h0=h0, scale=0.5)

    def loss(args, h0_):
        o, hT = oracle.kda_forward(*args, h0=h0_, scale=0.5)
        return float((o * do).sum() + (hT * dhT).sum())

    step = 2.0 ** -12
    for which, name in enumerate(NAMES):
        for trial in range(3):
            shape = h0.shape if which == 5 else arrs[which].shape
            direction = rng.choice([-1.0, 1.0], size=shape)
            plus, minus, hp, hm = list(arrs), list(arrs), h0, h0
            if which == 5:
                hp, hm = h0 + step * direction, h0 - step * direction
            else:
                plus[which] = arrs[which] + step * direction
                minus[which] = arrs[which] - step * direction
            num = (loss(plus, hp) - loss(minus, hm)) / (2 * step)
            ana = float((grads[name] * direction).sum())
            scale_ = np.abs(grads[name]).sum()
            assert abs(num - ana) < 1e-5 * scale_, (name, trial, num, ana)


def test_one_token_from_zero_state_closed_form():
    """T = 1, S_0 = 0: S_1 = beta k v^T and o = scale beta (q.k) v, so
    dq = scale beta (v.do) k,  dk = scale beta (v.do) q + beta dhT v,  dv = scale beta (q.k) do + beta dhT^T k,
    dbeta = scale (q.k)(v.do) + k^T dhT v,  dlog_alpha = 0 (nothing to decay)."""
    rng = np.random.default_rng(103)
    dk, dv = 5, 3
    q, k, v, g, b = _inputs(rng, 1, 1, 1, dk, dv)
    do = rng.standard_normal((1, 1, 1, dv))
    dhT = rng.standard_normal((1, 1, dk, dv))
    scale = 1.3
    gr = oracle.kda_backward(q, k, v, g, b, do, dhT=dhT, scale=scale)
    qq, kk, vv, bb = (x[0, 0, 0].astype(np.float64) for x in (q, k, v, b))
    d, D = do[0, 0, 0], dhT[0, 0]
    np.testing.assert_allclose(gr["dq"][0, 0, 0], scale * bb * (vv @ d) * kk, rtol=1e-13)
    np.testing.assert_allclose(gr["dk"][0, 0, 0], scale * bb * (vv @ d) * qq + bb * D @ vv, rtol=1e-13)
    np.testing.assert_allclose(gr["dv"][0, 0, 0], scale * bb * (qq @ kk) * d + bb * D.T @ kk, rtol=1e-13)
    np.testing.assert_allclose(gr["dbeta"][0, 0, 0], scale * (qq @ kk) * (vv @ d) + kk @ D @ vv, rtol=1e-13)
    assert np.abs(gr["dlog_alpha"]).max() == 0.0


def test_pure_decay_closed_form():
    """beta = 0: S_t = Diag(prod alpha) S_0 and o_t = scale S_t^T q_t.  Then
    dlog_alpha_t[c] = sum over s >= t of scale q_s[c] (S_s do_s)[c] + (S_T . dhT) row sums, and
    dh0 = sum_t Diag(prod_{<=t} alpha) scale q_t do_t^T + Diag(prod_all alpha) dhT."""
    rng = np.random.default_rng(104)
    T, dk, dv = 6, 4, 3
    q, k, v, g, b = _inputs(rng, 1, T, 1, dk, dv)
    b[:] = 0
    h0 = rng.standard_normal((1, 1, dk, dv)).astype(np.float32)
    do = rng.standard_normal((1, T, 1, dv))
    dhT = rng.standard_normal((1, 1, dk, dv))
    gr = oracle.kda_backward(q, k, v, g, b, do, dhT=dhT, h0=h0, scale=2.0)
    G = np.cumsum(g[0, :, 0].astype(np.float64), axis=0)
    S0 = h0[0, 0].astype(np.float64)
    per_tok = np.stack([2.0 * q[0, t, 0] * ((np.exp(G[t])[:, None] * S0) @ do[0, t, 0]) for t in range(T)])
    tail = ((np.exp(G[-1])[:, None] * S0) * dhT[0, 0]).sum(axis=1)
    want = per_tok[::-1].cumsum(axis=0)[::-1] + tail
    np.testing.assert_allclose(gr["dlog_alpha"][0, :, 0], want, rtol=1e-12, atol=1e-14)
    dh0 = sum(np.exp(G[t])[:, None] * 2.0 * np.outer(q[0, t, 0], do[0, t, 0]) for t in range(T))
    dh0 = dh0 + np.exp(G[-1])[:, None] * dhT[0, 0]
    np.testing.assert_allclose(gr["dh0"][0, 0], dh0, rtol=1e-12)
    assert np.abs(gr["dk"]).max() == 0 and np.abs(gr["dv"]).max() == 0


def test_euler_identities_at_full_head_size():
    """o and hT are linear in q (o only), and jointly linear in (v, h0): for a function that is
    homogeneous of degree one in x, <grad_x, x> equals the function.  d_k = d_v = 128, T = 150."""
    rng = np.random.default_rng(105)
    B, T, H, d = 1, 150, 2, 128
    q, k, v, g, b = _inputs(rng, B, T, H, d, d)
    h0 = rng.standard_normal((B, H, d, d)).astype(np.float32)
    do = rng.standard_normal((B, T, H, d))
    dhT = rng.standard_normal((B, H, d, d))
    o, hT = oracle.kda_forward(q, k, v, g, b, h0=h0, scale=d ** -0.5)
    gr = oracle.kda_backward(q, k, v, g, b, do, dhT=dhT, h0=h0, scale=d ** -0.5)
    lo, lh = (o * do).sum(), (hT * dhT).sum()
    assert abs((gr["dq"] * q).sum() - lo) < 1e-10 * abs(lo)
    assert abs((gr["dv"] * v).sum() + (gr["dh0"] * h0).sum() - (lo + lh)) < 1e-10 * (abs(lo) + abs(lh))


def test_packed_batch_equals_separate_calls_and_stray_tokens_get_zero():
    rng = np.random.default_rng(106)
    lens = [7, 0, 33, 1]
    cu = np.concatenate([[0], np.cumsum(lens)])
    T = int(cu[-1]) + 3                                   # three tokens belong to nobody
    H, dk, dv = 2, 4, 6
    q, k, v, g, b = _inputs(rng, 1, T, H, dk, dv)
    h0 = rng.standard_normal((len(lens), H, dk, dv)).astype(np.float32)
    do = rng.standard_normal((1, T, H, dv))
    dhT = rng.standard_normal((len(lens), H, dk, dv))
    gr = oracle.kda_backward(q, k, v, g, b, do, dhT=dhT, h0=h0, cu_seqlens=cu)
    for n, L in enumerate(lens):
        s, e = int(cu[n]), int(cu[n + 1])
        one = oracle.kda_backward(q[:, s:e], k[:, s:e], v[:, s:e], g[:, s:e], b[:, s:e], do[:, s:e],
                                  dhT=dhT[n:n + 1], h0=h0[n:n + 1])
        for name in NAMES[:5]:
            np.testing.assert_array_equal(gr[name][:, s:e], one[name])
        np.testing.assert_array_equal(gr["dh0"][n], one["dh0"][0])
    for name in NAMES[:5]:
        assert np.abs(gr[name][:, int(cu[-1]):]).max() == 0.0
    # an empty sequence hands its final-state gradient straight to its initial state
    np.testing.assert_array_equal(gr["dh0"][1], dhT[1])


def test_planted_mistakes_in_a_reverse_pass_are_caught_by_the_finite_difference_pin():
    """Sanity of the pins themselves: a numpy reverse pass with one plausible mistake at a time (a dropped
    term, a wrong sign, a missing decay, the undecayed state, the old state in place of the new one) is compared with central differences of the chunkwise forward exactly as the first pin does;
    the faithful version passes at 2e-7, every planted version misses some gradient by more than 1e-3."""
    rng = np.random.default_rng(107)
    T, dk, dv = 9, 3, 4
    q, k, v, g, b = (x[0, :, 0].astype(np.float64) for x in _inputs(rng, 1, T, 1, dk, dv))
    S0 = rng.standard_normal((dk, dv))
    do = rng.standard_normal((T, dv))
    dST = rng.standard_normal((dk, dv))

    def reverse(mistake=None):
        states = [S0]
        for t in range(T):
            Sp = np.exp(g[t])[:, None] * states[-1]
            states.append(Sp + b[t] * np.outer(k[t], v[t] - Sp.T @ k[t]))
        D = dST.copy()
        out = {n: np.zeros_like(x) for n, x in (("dq", q), ("dk", k), ("dv", v), ("dlog_alpha", g), ("dbeta", b))}
        for t in range(T - 1, -1, -1):
            a = np.exp(g[t])[:, None]
            Sp = a * states[t]
            u = v[t] - Sp.T @ k[t]
            St = states[t] if mistake == "old_state_in_dq" else states[t + 1]
            D = D + np.outer(q[t], do[t])
            out["dq"][t] = St @ do[t]
            out["dbeta"][t] = k[t] @ D @ u
            du = b[t] * (D.T @ k[t])
            out["dv"][t] = du
            corr = 0.0 if mistake == "dropped_correction_in_dk" else Sp @ du
            out["dk"][t] = b[t] * (D @ u) + (corr if mistake == "wrong_sign_in_dk" else -corr)
            Dp = D if mistake == "dropped_rank_one_in_dS" else D - np.outer(k[t], du)
            out["dlog_alpha"][t] = (Dp * (states[t] if mistake == "undecayed_state_in_dlog_alpha" else Sp)).sum(axis=1)
            D = Dp if mistake == "no_decay_of_dS" else a * Dp
        out["dh0"] = D
        return out

    def loss(args):
        o, hT = kda_chunkwise(*[x[None, :, None] for x in args[:5]], h0=args[5][None, None], C=4)
        return float((o[0, :, 0] * do).sum() + (hT[0, 0] * dST).sum())

    base = [q, k, v, g, b, S0]
    h = 1e-6
    numeric = {}
    for which, name in enumerate(NAMES):
        num = np.zeros_like(base[which])
        for idx in np.ndindex(*base[which].shape):
            plus = [x.copy() for x in base]
            minus = [x.copy() for x in base]
            plus[which][idx] += h
            minus[which][idx] -= h
            num[idx] = (loss(plus) - loss(minus)) / (2 * h)
        numeric[name] = num

    def worst(grads):
        return max(np.abs(grads[n] - numeric[n]).max() / np.abs(numeric[n]).max() for n in NAMES)

    assert worst(reverse()) < 2e-7
    for mistake in ("old_state_in_dq", "dropped_correction_in_dk", "wrong_sign_in_dk", "dropped_rank_one_in_dS",
                    "undecayed_state_in_dlog_alpha", "no_decay_of_dS"):
        assert worst(reverse(mistake)) > 1e-3, mistake
