"""Pins for the backward oracle (CPU only).  ``oracle.scan_bwd`` differentiates the recurrence of Sec. 3.1.3 step by
step; it is checked against things other than itself: central finite differences of the (separately pinned) forward
oracle, the closed-form gradients of plain causal linear attention it must reduce to, the single-step case worked by
hand, and the chaining of cotangents through a split sequence."""
import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(4321)


def _case(B, T, H, dk, dv, with_beta=True, with_s0=True, rng=RNG):
    f = np.float32
    q = rng.standard_normal((B, T, H, dk)).astype(f)
    k = rng.standard_normal((B, T, H, dk)).astype(f)
    v = rng.standard_normal((B, T, H, dv)).astype(f)
    la = (-np.abs(rng.standard_normal((B, T, H, dk))) * 0.7).astype(f)
    beta = rng.uniform(0.1, 1.0, (B, T, H, dv)).astype(f) if with_beta else None
    S0 = rng.standard_normal((B, H, dk, dv)).astype(f) if with_s0 else None
    return q, k, v, la, beta, S0


def _loss(q, k, v, la, beta, S0, Wo, Ws):
    o, S_T = oracle.scan(q, k, v, la, beta, S0)
    return float((o * Wo).sum() + (S_T * Ws).sum())


def test_matches_central_finite_differences_in_every_argument():
    """L = <Wo, o> + <Ws, S_T>; dL/dx by the backward oracle against (L(x+h) - L(x-h)) / 2h of the forward oracle.
    Perturbations are multiples of 2^-10 so that the perturbed inputs stay exact in float32."""
    B, T, H, dk, dv = 1, 70, 2, 3, 4          # T spans two of the oracle's 64-step segments
    q, k, v, la, beta, S0 = _case(B, T, H, dk, dv)
    q, k, v, la, beta, S0 = [np.round(x * 256) / 256 for x in (q, k, v, la, beta, S0)]      # 8 fractional bits
    q, k, v, la, beta, S0 = [x.astype(np.float32) for x in (q, k, v, la, beta, S0)]
    Wo = RNG.standard_normal((B, T, H, dv))
    Ws = RNG.standard_normal((B, H, dk, dv))
    g = oracle.scan_bwd(q, k, v, la, beta, S0, Wo, Ws)
    args = {"q": q, "k": k, "v": v, "la": la, "beta": beta, "S0": S0}
    names = {"q": "dq", "k": "dk", "v": "dv", "la": "dlog_alpha", "beta": "dbeta", "S0": "dS0"}
    h = 2.0 ** -10
    for name, arr in args.items():
        flat = arr.reshape(-1)
        for idx in RNG.choice(flat.size, size=12, replace=False):
            keep = flat[idx]
            flat[idx] = keep + h
            up = _loss(args["q"], args["k"], args["v"], args["la"], args["beta"], args["S0"], Wo, Ws)
            flat[idx] = keep - h
            dn = _loss(args["q"], args["k"], args["v"], args["la"], args["beta"], args["S0"], Wo, Ws)
            flat[idx] = keep
            fd = (up - dn) / (2 * h)
            got = g[names[name]].reshape(-1)[idx]
            assert abs(got - fd) <= 1e-5 * max(1.0, abs(fd)), (name, idx, got, fd)


def test_reduces_to_linear_attention_gradients():
    """alpha = 1, beta = 1, S0 = 0: o = tril(Q K^T) V, so with M = tril(ones):
    dQ = (M .* dO V^T) K,  dK = (M .* dO V^T)^T Q,  dV = (M .* Q K^T)^T dO  (Sec. 2, identity-map linear attention)."""
    B, T, H, dk, dv = 1, 29, 1, 5, 6
    q, k, v, _, _, _ = _case(B, T, H, dk, dv, with_beta=False, with_s0=False)
    la = np.zeros((B, T, H, dk), np.float32)
    dO = RNG.standard_normal((B, T, H, dv))
    g = oracle.scan_bwd(q, k, v, la, None, None, dO)
    Q, K, V, D = [x[0, :, 0].astype(np.float64) for x in (q, k, v, dO)]
    M = np.tril(np.ones((T, T)))
    W = M * (D @ V.T)
    np.testing.assert_allclose(g["dq"][0, :, 0], W @ K, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(g["dk"][0, :, 0], W.T @ Q, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(g["dv"][0, :, 0], (M * (Q @ K.T)).T @ D, rtol=1e-12, atol=1e-12)
    assert g["dbeta"] is None
    # d/dlog_alpha at alpha = 1: every earlier write (and nothing else, S0 = 0) passes through gate t on its way to a
    # later or equal query: sum_{i < t <= s} q_s[n] k_i[n] (dO_s . V_i)
    ref = np.zeros((T, dk))
    G = D @ V.T
    for t in range(T):
        for s in range(t, T):
            for i in range(t):
                ref[t] += Q[s] * K[i] * G[s, i]
    np.testing.assert_allclose(g["dlog_alpha"][0, :, 0], ref, rtol=1e-11, atol=1e-11)


def test_single_step_by_hand():
    """T = 1: S_1 = a .* S_0 + k^T u, o = q S_1.  Everything follows from two lines of calculus."""
    dk, dv = 3, 2
    q, k, v, la, beta, S0 = _case(1, 1, 1, dk, dv)
    dO = RNG.standard_normal((1, 1, 1, dv))
    dS = RNG.standard_normal((1, 1, dk, dv))
    g = oracle.scan_bwd(q, k, v, la, beta, S0, dO, dS)
    Q, K, V, L, Bt = [x[0, 0, 0].astype(np.float64) for x in (q, k, v, la, beta)]
    S_0, d_o, d_s = S0[0, 0].astype(np.float64), dO[0, 0, 0], dS[0, 0]
    a, u = np.exp(L), Bt * V
    S1 = a[:, None] * S_0 + np.outer(K, u)
    G = np.outer(Q, d_o) + d_s
    np.testing.assert_allclose(g["dq"][0, 0, 0], S1 @ d_o, rtol=1e-13)
    np.testing.assert_allclose(g["dk"][0, 0, 0], G @ u, rtol=1e-13)
    np.testing.assert_allclose(g["dv"][0, 0, 0], Bt * (K @ G), rtol=1e-13)
    np.testing.assert_allclose(g["dbeta"][0, 0, 0], V * (K @ G), rtol=1e-13)
    np.testing.assert_allclose(g["dlog_alpha"][0, 0, 0], a * (G * S_0).sum(1), rtol=1e-13)
    np.testing.assert_allclose(g["dS0"][0, 0], a[:, None] * G, rtol=1e-13)


def test_split_sequence_chains_the_state_cotangent():
    """Backward over [0, T) equals backward over [T1, T) followed by backward over [0, T1) fed with the first one's dS0
    (the chain rule through the carried state), with the second half started from the first half's final state."""
    B, T, H, dk, dv, T1 = 2, 90, 2, 4, 3, 37
    q, k, v, la, beta, S0 = _case(B, T, H, dk, dv)
    dO = RNG.standard_normal((B, T, H, dv))
    dS = RNG.standard_normal((B, H, dk, dv))
    whole = oracle.scan_bwd(q, k, v, la, beta, S0, dO, dS)
    _, S_mid = oracle.scan(q[:, :T1], k[:, :T1], v[:, :T1], la[:, :T1], beta[:, :T1], S0)
    # second half from the exact mid state (initial states are taken in double)
    second = oracle.scan_bwd(q[:, T1:], k[:, T1:], v[:, T1:], la[:, T1:], beta[:, T1:], S_mid, dO[:, T1:], dS)
    first = oracle.scan_bwd(q[:, :T1], k[:, :T1], v[:, :T1], la[:, :T1], beta[:, :T1], S0, dO[:, :T1], second["dS0"])
    for name in ("dq", "dk", "dv", "dlog_alpha", "dbeta"):
        np.testing.assert_allclose(np.concatenate([first[name], second[name]], axis=1), whole[name], rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(first["dS0"], whole["dS0"], rtol=1e-10, atol=1e-11)


def test_closed_gate_blocks_the_gradient():
    """alpha_t = 0 at one step: nothing before it can influence later outputs, so dq after the reset does not depend on
    earlier tokens' cotangents and the gradients of earlier k, v come only from outputs before the reset."""
    B, T, H, dk, dv, cut = 1, 20, 1, 3, 4, 11
    q, k, v, la, beta, S0 = _case(B, T, H, dk, dv)
    la[:, cut] = -np.inf
    dO = RNG.standard_normal((B, T, H, dv))
    g = oracle.scan_bwd(q, k, v, la, beta, S0, dO)
    dO2 = dO.copy()
    dO2[:, cut:] = 0.0                      # cotangents after the reset cannot reach tokens before it
    g2 = oracle.scan_bwd(q, k, v, la, beta, S0, dO2)
    for name in ("dk", "dv", "dbeta", "dlog_alpha"):
        np.testing.assert_allclose(g[name][:, :cut], g2[name][:, :cut], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(g["dS0"], g2["dS0"], rtol=1e-12, atol=1e-13)
    assert np.all(g["dlog_alpha"][:, cut] == 0.0)      # d/dlog_alpha = alpha * (...) vanishes with alpha


def test_mutations_of_the_backward_rules_fail_the_finite_difference_pin():
    """Plausible mistakes (own gate applied to the token's own write, the output taken from the state before the update)
    change dL/dk by far more than the finite-difference tolerance: the pin can tell them apart."""
    B, T, H, dk, dv = 1, 6, 1, 2, 2
    q, k, v, la, beta, S0 = _case(B, T, H, dk, dv)
    Wo = RNG.standard_normal((B, T, H, dv))
    g = oracle.scan_bwd(q, k, v, la, beta, S0, Wo)

    def wrong_dk(kind):
        # hand-written variants of dk_t = u_t G_t^T with a wrong G_t
        a = np.exp(la[0, :, 0].astype(np.float64))
        Q, Bt, V = q[0, :, 0].astype(np.float64), beta[0, :, 0].astype(np.float64), v[0, :, 0].astype(np.float64)
        D = Wo[0, :, 0]
        G = np.zeros((dk, dv))
        out = np.zeros((T, dk))
        for t in range(T - 1, -1, -1):
            if kind == "pre_update_output":      # o_t = q_t S_{t-1}: the token's own cotangent is missing from G_t
                out[t] = G @ (Bt[t] * V[t])
                G = a[t][:, None] * (G + np.outer(Q[t], D[t]))
            else:                                 # own gate applied to the own write
                G = G + np.outer(Q[t], D[t])
                out[t] = a[t] * (G @ (Bt[t] * V[t]))
                G = a[t][:, None] * G
        return out

    for kind in ("pre_update_output", "own_gate_on_own_write"):
        assert np.abs(wrong_dk(kind) - g["dk"][0, :, 0]).max() > 1e-2


def test_value_gate_as_pre_activation():
    """beta = sigmoid(z_beta) (Sec. 3.1.2): the z_beta form of the backward oracle against central finite differences of the
    z_beta form of the forward oracle in z_beta, and against the chain rule on the plain form for every other gradient."""
    B, T, H, dk, dv = 1, 37, 2, 3, 5
    q, k, v, la, _, S0 = _case(B, T, H, dk, dv)
    z = (np.round(RNG.standard_normal((B, T, H, dv)) * 2 * 256) / 256).astype(np.float32)
    q, k, v, la, S0 = [(np.round(x * 256) / 256).astype(np.float32) for x in (q, k, v, la, S0)]
    Wo = RNG.standard_normal((B, T, H, dv))
    Ws = RNG.standard_normal((B, H, dk, dv))
    g = oracle.scan_bwd(q, k, v, la, None, S0, Wo, Ws, z_beta=z)
    assert "dbeta" not in g

    def loss(zz):
        o, S_T = oracle.scan(q, k, v, la, None, S0, z_beta=zz)
        return float((o * Wo).sum() + (S_T * Ws).sum())

    h = 2.0 ** -10
    flat = z.reshape(-1)
    for idx in RNG.choice(flat.size, size=16, replace=False):
        keep = flat[idx]
        flat[idx] = keep + h
        up = loss(z)
        flat[idx] = keep - h
        down = loss(z)
        flat[idx] = keep
        fd = (up - down) / (2 * h)
        assert abs(g["dz_beta"].reshape(-1)[idx] - fd) <= 1e-5 * max(1.0, abs(fd)), (idx, g["dz_beta"].reshape(-1)[idx], fd)
    # the other gradients are those of the plain form at beta = sigmoid(z) (the float32 rounding of beta is all that differs)
    beta = (1.0 / (1.0 + np.exp(-z.astype(np.float64))))
    plain = oracle.scan_bwd(q, k, v, la, beta.astype(np.float32), S0, Wo, Ws)
    for name in ("dq", "dk", "dv", "dlog_alpha", "dS0"):
        assert np.abs(g[name] - plain[name]).max() <= 1e-6 * max(1.0, np.abs(plain[name]).max()), name
    assert np.abs(g["dz_beta"] - plain["dbeta"] * beta * (1 - beta)).max() <= 1e-6 * np.abs(g["dz_beta"]).max()
    # a saturated gate passes no gradient to its pre-activation
    z_sat = z.copy(); z_sat[:, 5] = 60.0; z_sat[:, 6] = -60.0
    gs = oracle.scan_bwd(q, k, v, la, None, S0, Wo, Ws, z_beta=z_sat)
    assert np.abs(gs["dz_beta"][:, 5:7]).max() < 1e-20
