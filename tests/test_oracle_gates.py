"""Pins for the oracle's DDTS gate front-end (CPU only): closed forms, the identities the paper states, the
selection property of Proposition 1, and the role of the temperature."""
import os

import numpy as np

import oracle


def _gates(z_g, z_tau, k=None, q=None, z_beta=None):
    z_g = np.atleast_2d(np.asarray(z_g, np.float32))
    z_tau = np.atleast_2d(np.asarray(z_tau, np.float32))
    k = np.ones_like(z_g) if k is None else np.atleast_2d(np.asarray(k, np.float32))
    q = np.ones_like(z_g) if q is None else np.atleast_2d(np.asarray(q, np.float32))
    return oracle.ddts_gates(z_g, z_tau, z_beta, q, k)


def _alpha_hat(k_out, k):
    """alpha_hat recovered from k_out = alpha_hat .* k / ||k||."""
    k = np.atleast_2d(np.asarray(k, np.float64))
    return k_out * np.linalg.norm(k, axis=-1, keepdims=True) / k


def test_closed_form_values(golden_dir):
    rows = [list(map(float, l.split())) for l in open(os.path.join(golden_dir, "ddts_gates_closed_forms.txt"))
            if l.strip() and not l.startswith("#")]
    for z_g, z_tau, alpha, alpha_hat in rows:
        la, _, _, ko = _gates([[z_g]], [[z_tau]])
        # the inputs pass through float32, so compare at float32 resolution
        np.testing.assert_allclose(np.exp(la[0, 0]), alpha, rtol=3e-7)
        np.testing.assert_allclose(ko[0, 0], alpha_hat, rtol=3e-7)      # k = 1, ||k|| = 1


def test_decay_identity_and_ranges():
    """exp(-softplus(z)) = 1 - sigmoid(z) (stated under the gate definition), hence alpha in [0, 1] at tau = 1;
    alpha_hat >= 0 and exceeds 1 where g > 1."""
    z = np.linspace(-30, 30, 241).astype(np.float32)[None]
    la, _, _, ko = _gates(z, np.full_like(z, 60.0))            # tau = 1
    one_minus_sig = 1 / (1 + np.exp(z.astype(np.float64)))     # 1 - sigmoid(z) = sigmoid(-z), without cancellation
    np.testing.assert_allclose(np.exp(la), one_minus_sig, rtol=1e-12)
    np.testing.assert_allclose(np.exp(la)[np.abs(z) < 5], (1 - 1 / (1 + np.exp(-z.astype(np.float64))))[np.abs(z) < 5], rtol=1e-12)
    z_tau = np.random.default_rng(0).standard_normal(z.shape).astype(np.float32)
    la, _, _, ko = _gates(z, z_tau)
    assert (la <= 0).all() and (np.exp(la) <= 1).all()
    ah = _alpha_hat(ko, np.ones_like(z))
    assert (ah >= 0).all() and (ah[z > 2] > 1).all() and (ah[z < -2] < 1).all()


def test_selection_property():
    """Proposition 1: the decay of the old state and the gate on the new input move in opposite directions with the
    selection pre-activation (d alpha / d z_g < 0 < d alpha_hat / d z_g), for any temperature."""
    rng = np.random.default_rng(1)
    z_g = rng.uniform(-4, 4, (1, 64)).astype(np.float32)
    z_tau = rng.uniform(-3, 3, (1, 64)).astype(np.float32)
    h = np.float32(1e-2)
    la0, _, _, k0 = _gates(z_g, z_tau)
    la1, _, _, k1 = _gates(z_g + h, z_tau)
    assert (np.exp(la1) < np.exp(la0)).all()
    assert (k1 > k0).all()


def test_temperature_controls_sharpness():
    """A smaller tau makes alpha change more slowly with g (Sec. 3.1.2, temperature gate)."""
    z_g = np.array([[-1.0, 0.0, 0.3]], np.float32)              # g < 1
    h = np.float32(1e-2)
    slopes = []
    for z_tau in (-2.0, 0.0, 2.0):
        zt = np.full_like(z_g, z_tau)
        a0 = np.exp(_gates(z_g, zt)[0])
        a1 = np.exp(_gates(z_g + h, zt)[0])
        slopes.append(np.abs(a1 - a0))
    assert (slopes[0] < slopes[1]).all() and (slopes[1] < slopes[2]).all()


def test_key_normalisation_query_scale_and_value_gate():
    rng = np.random.default_rng(2)
    M, dk, dv = 7, 16, 12
    z_g, z_tau, q, k = (rng.standard_normal((M, dk)).astype(np.float32) for _ in range(4))
    z_beta = rng.standard_normal((M, dv)).astype(np.float32)
    la, beta, qo, ko = oracle.ddts_gates(z_g, z_tau, z_beta, q, k)
    g = np.log1p(np.exp(z_g.astype(np.float64)))
    tau = 1 / (1 + np.exp(-z_tau.astype(np.float64)))
    np.testing.assert_allclose(la, -g * tau, rtol=1e-12)
    np.testing.assert_allclose(np.linalg.norm(ko / g ** tau, axis=-1), 1.0, rtol=1e-12)      # unit keys before the gate
    np.testing.assert_allclose(ko / g ** tau * np.linalg.norm(k.astype(np.float64), axis=-1, keepdims=True), k, rtol=1e-12)
    np.testing.assert_allclose(qo, q / 4.0, rtol=1e-15)                                      # 1 / sqrt(16)
    np.testing.assert_allclose(beta, 1 / (1 + np.exp(-z_beta.astype(np.float64))), rtol=1e-12)
    np.testing.assert_allclose(beta + oracle.ddts_gates(z_g, z_tau, -z_beta, q, k)[1], 1.0, rtol=1e-12)
    # a zero key stays zero instead of dividing by zero
    k[3] = 0
    assert np.all(oracle.ddts_gates(z_g, z_tau, None, q, k)[3][3] == 0)


def test_gates_feed_the_recurrence():
    """End to end on the CPU: gates -> recurrence equals the block recurrence written with alpha and alpha_hat
    explicitly (first form of the transition in Sec. 3.1.1)."""
    rng = np.random.default_rng(3)
    T, dk, dv = 9, 4, 3
    z_g, z_tau, q, k = (rng.standard_normal((1, T, 1, dk)).astype(np.float32) for _ in range(4))
    z_beta = rng.standard_normal((1, T, 1, dv)).astype(np.float32)
    v = rng.standard_normal((1, T, 1, dv)).astype(np.float32)
    la, beta, qo, ko = oracle.ddts_gates(z_g, z_tau, z_beta, q, k)
    f32 = lambda x: x.astype(np.float32)
    o, _ = oracle.scan(f32(qo), f32(ko), v, f32(la), f32(beta))
    # explicit form with the same float32-rounded gate values
    a, kk, qq, bb = np.exp(f32(la).astype(np.float64)), f32(ko).astype(np.float64), f32(qo).astype(np.float64), f32(beta).astype(np.float64)
    S = np.zeros((dk, dv))
    for t in range(T):
        S = a[0, t, 0][:, None] * S + np.outer(kk[0, t, 0], bb[0, t, 0] * v[0, t, 0])
        np.testing.assert_allclose(o[0, t, 0], qq[0, t, 0] @ S, rtol=1e-12, atol=1e-14)


def test_block_output_stage_closed_forms(golden_dir):
    """Feed-through and output gate (Sec. 3.1.3): hand-worked values, the no-op cases, and the two activations' limits."""
    import os
    vals = None
    with open(os.path.join(golden_dir, "block_output_closed_forms.txt")) as fh:
        for line in fh:
            if line.startswith("block_output:"):
                vals = [float(x) for x in line.split(":")[1].split()]
    o = np.array([[[3.0]]])
    x = np.array([[[4.0]]], np.float32)
    d = np.array([[0.5]], np.float32)
    z0 = np.zeros((1, 1, 1), np.float32)
    assert oracle.block_output(o, x, d, z0, "sigmoid")[0, 0, 0] == vals[0]
    assert oracle.block_output(o, x, d, z0, "silu")[0, 0, 0] == vals[1]
    o2 = np.array([[[-2.0]]])
    z3 = np.full((1, 1, 1), np.log(3.0), np.float32)
    z3d = float(z3[0, 0, 0])                                  # the float32 value the oracle sees
    sg = 1.0 / (1.0 + np.exp(-z3d))
    np.testing.assert_allclose(oracle.block_output(o2, None, None, z3, "sigmoid")[0, 0, 0], vals[2], rtol=1e-7)
    np.testing.assert_allclose(oracle.block_output(o2, None, None, z3, "silu")[0, 0, 0], vals[3], rtol=1e-7)
    np.testing.assert_allclose(oracle.block_output(o2, None, None, z3, "silu")[0, 0, 0], -2.0 * z3d * sg, rtol=1e-15)
    # nothing given: identity; per-head d broadcasts over rows; saturated gates
    rng = np.random.default_rng(5)
    o = rng.standard_normal((7, 3, 4))
    assert np.array_equal(oracle.block_output(o), o)
    xp = rng.standard_normal((7, 3, 4)).astype(np.float32)
    dd = rng.standard_normal((3, 4)).astype(np.float32)
    np.testing.assert_allclose(oracle.block_output(o, xp, dd), o + dd[None].astype(np.float64) * xp, rtol=1e-15)
    big = np.full((7, 3, 4), 50.0, np.float32)
    np.testing.assert_allclose(oracle.block_output(o, None, None, big, "sigmoid"), o, rtol=1e-15)
    np.testing.assert_allclose(oracle.block_output(o, None, None, big, "silu"), 50.0 * o, rtol=1e-15)
    assert np.all(oracle.block_output(o, None, None, -big, "sigmoid") == o * (np.exp(-50.0) / (1.0 + np.exp(-50.0))))


def _numpy_block_recurrence(q, k, v, z_g, z_tau, z_beta, S0):
    """The block equation of Sec. 3.1.3 written out in numpy float64 for tiny inputs (brute force, token by token)."""
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    f = lambda a: np.asarray(a, np.float64)
    q, k, v, z_g, z_tau = f(q), f(k), f(v), f(z_g), f(z_tau)
    g = np.logaddexp(0.0, z_g)
    tau = 1.0 / (1.0 + np.exp(-z_tau))
    bh = np.ones_like(v) if z_beta is None else 1.0 / (1.0 + np.exp(-f(z_beta)))
    o = np.zeros((B, T, H, dv))
    S = np.zeros((B, H, dk, dv)) if S0 is None else f(S0).copy()
    for b in range(B):
        for h in range(H):
            for t in range(T):
                kn = k[b, t, h] / max(np.linalg.norm(k[b, t, h]), 1e-12)
                S[b, h] = np.exp(-g[b, t, h] * tau[b, t, h])[:, None] * S[b, h] + \
                    np.outer(g[b, t, h] ** tau[b, t, h] * kn, bh[b, t, h] * v[b, t, h])
                o[b, t, h] = (q[b, t, h] / np.sqrt(dk)) @ S[b, h]
    return o, S


def test_gated_recurrence_brute_force_composition_and_closed_form():
    rng = np.random.default_rng(17)
    B, T, H, dk, dv = 2, 9, 2, 4, 3
    d = {n: rng.standard_normal((B, T, H, dk)).astype(np.float32) for n in ("q", "k", "z_g", "z_tau")}
    v = rng.standard_normal((B, T, H, dv)).astype(np.float32)
    zb = rng.standard_normal((B, T, H, dv)).astype(np.float32)
    S0 = rng.standard_normal((B, H, dk, dv))
    for z_beta, s0 in ((zb, S0), (None, None)):
        o, S_T = oracle.scan_gated(d["q"], d["k"], v, d["z_g"], d["z_tau"], z_beta, s0)
        o_n, S_n = _numpy_block_recurrence(d["q"], d["k"], v, d["z_g"], d["z_tau"], z_beta, s0)
        np.testing.assert_allclose(o, o_n, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(S_T, S_n, rtol=1e-12, atol=1e-13)
    # decode steps chain to the scan
    S = S0.copy()
    o_steps = []
    for t in range(T):
        o_t, S = oracle.step_gated(d["q"][:, t], d["k"][:, t], v[:, t], d["z_g"][:, t], d["z_tau"][:, t], zb[:, t], S)
        o_steps.append(o_t)
    o, S_T = oracle.scan_gated(d["q"], d["k"], v, d["z_g"], d["z_tau"], zb, S0)
    assert np.array_equal(np.stack(o_steps, axis=1), o) and np.array_equal(S, S_T)
    # closed form: tau -> 1 (z_tau = 40), g = 1 (z_g = log(e - 1)): decay 1/e, key gate 1; with k = q = e_1 * c and v = 1
    # the first state row is the geometric series and o_t = c / sqrt(dk) * (1 - e^-t) / (1 - 1/e)
    T2, dk2 = 12, 4
    zg1 = np.full((1, T2, 1, dk2), np.log(np.e - 1.0), np.float32)
    zt1 = np.full((1, T2, 1, dk2), 40.0, np.float32)
    e1 = np.zeros((1, T2, 1, dk2), np.float32)
    e1[..., 0] = 3.0                              # normalisation brings the key back to the unit vector
    ones = np.ones((1, T2, 1, 2), np.float32)
    o, S_T = oracle.scan_gated(e1, e1, ones, zg1, zt1, None, None)
    g_exact = np.logaddexp(0.0, np.float64(zg1[0, 0, 0, 0]))      # softplus of the float32 value, ~1
    gam = np.exp(-g_exact)
    t = np.arange(1, T2 + 1)
    np.testing.assert_allclose(o[0, :, 0, 0], 3.0 / 2.0 * g_exact * (1 - gam ** t) / (1 - gam), rtol=1e-9)
    assert np.all(S_T[0, 0, 1:] == 0)
    # zero key: the normalisation guard leaves it zero, nothing is written
    o, S_T = oracle.scan_gated(e1, np.zeros_like(e1), ones, zg1, zt1, None, None)
    assert np.all(o == 0) and np.all(S_T == 0)


def test_gated_recurrence_agrees_with_gate_front_end_then_scan():
    # the two-call pipeline (gates, rounded to float32, then the plain recurrence) reaches the same result up to that rounding
    rng = np.random.default_rng(23)
    B, T, H, dk, dv = 1, 40, 2, 8, 5
    d = {n: rng.standard_normal((B, T, H, dk)).astype(np.float32) for n in ("q", "k", "z_g", "z_tau")}
    v = rng.standard_normal((B, T, H, dv)).astype(np.float32)
    zb = rng.standard_normal((B, T, H, dv)).astype(np.float32)
    la, beta, qo, ko = oracle.ddts_gates(d["z_g"], d["z_tau"], zb, d["q"], d["k"])
    f = lambda a: a.astype(np.float32)
    o2, S2 = oracle.scan(f(qo), f(ko), v, f(la), f(beta))
    o1, S1 = oracle.scan_gated(d["q"], d["k"], v, d["z_g"], d["z_tau"], zb)
    np.testing.assert_allclose(o1, o2, rtol=0, atol=2e-6 * np.abs(o2).max())
    np.testing.assert_allclose(S1, S2, rtol=0, atol=2e-6 * np.abs(S2).max())
