"""Pins for the backward oracle of the gated scan (CPU only).  ``oracle.scan_gated_bwd`` differentiates the block's
recurrence through the DDTS gates (Sec. 3.1.2) and the pre-processing of q and k (Sec. 3.1.3).  It is checked against
things other than itself: central finite differences of the (separately pinned) forward oracle ``scan_gated`` in every
argument, the chain rule assembled from two other oracle functions (``scan_bwd`` on the outputs of ``ddts_gates``), the
behaviour at the key-norm guard, the opposite signs Proposition 1 gives the two key-side gates, and planted mistakes."""
import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(2718)


def _case(B, T, H, dk, dv, with_beta=True, with_s0=True, rng=RNG, bits=8):
    """Random inputs with `bits` fractional bits, so that +- 2^-10 perturbations stay exact in float32."""
    r = lambda shape, scale=1.0: (np.round(rng.standard_normal(shape) * scale * 2 ** bits) / 2 ** bits).astype(np.float32)
    return {"q": r((B, T, H, dk)), "k": r((B, T, H, dk)), "v": r((B, T, H, dv)), "z_g": r((B, T, H, dk)),
            "z_tau": r((B, T, H, dk)), "z_beta": r((B, T, H, dv), 1.5) if with_beta else None,
            "S0": r((B, H, dk, dv)) if with_s0 else None}


def _loss(a, Wo, Ws):
    o, S_T = oracle.scan_gated(a["q"], a["k"], a["v"], a["z_g"], a["z_tau"], a["z_beta"], a["S0"])
    return float((o * Wo).sum() + (S_T * Ws).sum())


NAMES = {"q": "dq", "k": "dk", "v": "dv", "z_g": "dz_g", "z_tau": "dz_tau", "z_beta": "dz_beta", "S0": "dS0"}


def _check_against_finite_differences(a, Wo, Ws, h, picks, tol):
    g = oracle.scan_gated_bwd(a["q"], a["k"], a["v"], a["z_g"], a["z_tau"], a["z_beta"], a["S0"], Wo, Ws)
    for name, arr in a.items():
        if arr is None:
            continue
        flat = arr.reshape(-1)
        for idx in RNG.choice(flat.size, size=min(picks, flat.size), replace=False):
            keep = flat[idx]
            flat[idx] = keep + h
            up = _loss(a, Wo, Ws)
            flat[idx] = keep - h
            dn = _loss(a, Wo, Ws)
            flat[idx] = keep
            fd = (up - dn) / (2 * h)
            got = g[NAMES[name]].reshape(-1)[idx]
            assert abs(got - fd) <= tol * max(1.0, abs(fd)), (name, idx, got, fd)
    return g


def test_matches_central_finite_differences_in_every_argument():
    """L = <Wo, o> + <Ws, S_T>; dL/dx by the backward oracle against (L(x+h) - L(x-h)) / 2h of the forward oracle."""
    B, T, H, dk, dv = 1, 70, 2, 3, 4          # T spans two of the oracle's 64-step segments
    a = _case(B, T, H, dk, dv)
    Wo = RNG.standard_normal((B, T, H, dv))
    Ws = RNG.standard_normal((B, H, dk, dv))
    _check_against_finite_differences(a, Wo, Ws, 2.0 ** -10, 14, 2e-5)


def test_without_value_gate_and_initial_state():
    a = _case(2, 9, 1, 4, 3, with_beta=False, with_s0=False)
    Wo = RNG.standard_normal((2, 9, 1, 3))
    Ws = RNG.standard_normal((2, 1, 4, 3))
    g = _check_against_finite_differences(a, Wo, Ws, 2.0 ** -10, 10, 2e-5)
    assert g["dz_beta"] is None


def test_chain_rule_through_the_gate_front_end():
    """The same gradients assembled from two other oracle functions: ``scan_bwd`` applied to the outputs of
    ``ddts_gates`` (log_alpha, folded key, scaled query, value gate), then the derivative of the gate map written out
    here.  The gate outputs pass through float32 on the way (``scan_bwd`` takes float32 inputs), hence 1e-5."""
    B, T, H, dk, dv = 2, 40, 2, 5, 6
    a = _case(B, T, H, dk, dv)
    dO = RNG.standard_normal((B, T, H, dv))
    dS = RNG.standard_normal((B, H, dk, dv))
    got = oracle.scan_gated_bwd(a["q"], a["k"], a["v"], a["z_g"], a["z_tau"], a["z_beta"], a["S0"], dO, dS)
    la, beta, qh, kh = oracle.ddts_gates(a["z_g"], a["z_tau"], a["z_beta"], a["q"], a["k"])
    inner = oracle.scan_bwd(qh.astype(np.float32), kh.astype(np.float32), a["v"], la.astype(np.float32), beta.astype(np.float32),
                            a["S0"], dO, dS)
    zg, zt, k64 = [a[n].astype(np.float64) for n in ("z_g", "z_tau", "k")]
    g = np.logaddexp(0.0, zg)
    tau = 1.0 / (1.0 + np.exp(-zt))
    w = g ** tau
    norm = np.sqrt((k64 ** 2).sum(-1, keepdims=True))
    dkh, dla = inner["dk"], inner["dlog_alpha"]
    dk = dkh * w / norm - k64 * (dkh * w * k64).sum(-1, keepdims=True) / norm ** 3
    dw = dkh * k64 / norm
    dg = -dla * tau + dw * tau * g ** (tau - 1.0)
    dtau = -dla * g + dw * w * np.log(g)
    ref = {"dq": inner["dq"] / np.sqrt(dk_ := float(dk.shape[-1])), "dk": dk, "dv": inner["dv"],
           "dz_g": dg / (1.0 + np.exp(-zg)), "dz_tau": dtau * tau * (1.0 - tau),
           "dz_beta": inner["dbeta"] * beta * (1.0 - beta), "dS0": inner["dS0"]}
    for name, r in ref.items():
        scale = np.abs(r).max()
        assert np.abs(got[name] - r).max() <= 1e-5 * scale, name


def test_key_norm_guard():
    """A key row whose norm lies below 1e-12 is divided by the guard, a constant: the map is then linear in that row, the
    term through the norm is absent, and finite differences with a step of the row's own size are exact."""
    B, T, H, dk, dv = 1, 6, 1, 4, 3
    a = _case(B, T, H, dk, dv)
    tiny = np.float32(2.0 ** -44)                       # 5.7e-14: the row's norm stays below the guard even when perturbed
    a["k"][0, 2, 0] = np.array([1, -2, 0, 1], np.float32) * tiny
    a["k"][0, 4, 0] = 0.0                               # a zero key: nothing written, still a finite gradient
    Wo = RNG.standard_normal((B, T, H, dv))
    Ws = RNG.standard_normal((B, H, dk, dv))
    g = oracle.scan_gated_bwd(a["q"], a["k"], a["v"], a["z_g"], a["z_tau"], a["z_beta"], a["S0"], Wo, Ws)
    assert np.isfinite(g["dk"]).all() and np.isfinite(g["dz_g"]).all()
    for t in (2, 4):
        for r in range(dk):
            keep = a["k"][0, t, 0, r]
            a["k"][0, t, 0, r] = keep + tiny
            up = _loss(a, Wo, Ws)
            a["k"][0, t, 0, r] = keep - tiny
            dn = _loss(a, Wo, Ws)
            a["k"][0, t, 0, r] = keep
            fd = (up - dn) / (2 * float(tiny))
            assert abs(g["dk"][0, t, 0, r] - fd) <= 1e-6 * max(1.0, abs(fd)), (t, r, g["dk"][0, t, 0, r], fd)
    # the guarded rows' gradient is dkhat .* w / 1e-12: no projection onto the key
    a2 = {n: (None if x is None else x.copy()) for n, x in a.items()}
    a2["k"][0, 2, 0] *= 2                                # still guarded: twice the key, same dk (linear map)
    g2 = oracle.scan_gated_bwd(a2["q"], a2["k"], a2["v"], a2["z_g"], a2["z_tau"], a2["z_beta"], a2["S0"], Wo, Ws)
    # (later steps see a different state, so only the last guarded row's own step is compared: t = 4 has k = 0 in both)
    np.testing.assert_allclose(g2["dk"][0, 4, 0], g["dk"][0, 4, 0], rtol=1e-9)


def test_proposition_one_signs_single_step():
    """T = 1, S0 = 0, one channel: o = q/sqrt(1) * g^tau * sign(k) * s v.  Raising z_g strengthens the write (alpha_hat grows,
    Proposition 1) while the decay it also strengthens has nothing to act on: d o / d z_g = o * tau * sigmoid(z_g) / g > 0
    for o > 0.  With S0 != 0 and k = 0 only the decay acts and the sign flips."""
    q = np.array([[[[1.0]]]], np.float32); k = np.array([[[[2.0]]]], np.float32); v = np.array([[[[3.0]]]], np.float32)
    zg = np.array([[[[0.5]]]], np.float32); zt = np.array([[[[-0.25]]]], np.float32)
    dO = np.ones((1, 1, 1, 1))
    g = oracle.scan_gated_bwd(q, k, v, zg, zt, None, None, dO)
    sp, tau = np.log1p(np.exp(0.5)), 1 / (1 + np.exp(0.25))
    o = sp ** tau * 3.0
    np.testing.assert_allclose(g["dz_g"].item(), o * tau / sp / (1 + np.exp(-0.5)), rtol=1e-12)
    np.testing.assert_allclose(g["dz_tau"].item(), o * np.log(sp) * tau * (1 - tau), rtol=1e-12)
    np.testing.assert_allclose(g["dk"].item(), 0.0, atol=1e-12)          # a one-channel key is normalised away entirely
    S0 = np.array([[[[4.0]]]], np.float32)
    g = oracle.scan_gated_bwd(q, np.zeros_like(k), v, zg, zt, None, S0, dO)
    a = np.exp(-sp * tau)
    np.testing.assert_allclose(g["dz_g"].item(), -a * 4.0 * tau / (1 + np.exp(-0.5)), rtol=1e-12)   # < 0: only the decay acts
    np.testing.assert_allclose(g["dS0"].item(), a, rtol=1e-12)


def test_planted_mistakes_fail_the_finite_difference_pin():
    """Plausible mistakes in the chain rule, planted in a numpy transcription of the per-step rule on a single step: each
    changes a gradient that the finite-difference pin above resolves (the pin's tolerance is 2e-5 relative)."""
    rng = np.random.default_rng(5)
    dk, dv = 4, 3
    a = _case(1, 1, 1, dk, dv, rng=rng)
    Wo = rng.standard_normal((1, 1, 1, dv))
    Ws = rng.standard_normal((1, 1, dk, dv))
    good = oracle.scan_gated_bwd(a["q"], a["k"], a["v"], a["z_g"], a["z_tau"], a["z_beta"], a["S0"], Wo, Ws)

    def by_hand(drop_norm_term=False, wrong_decay_sign=False, forget_alpha_hat=False):
        q, k, v, zg, zt, zb = [a[n][0, 0, 0].astype(np.float64) for n in ("q", "k", "v", "z_g", "z_tau", "z_beta")]
        S0 = a["S0"][0, 0].astype(np.float64)
        g, tau, s = np.logaddexp(0, zg), 1 / (1 + np.exp(-zt)), 1 / (1 + np.exp(-zb))
        al, w, n = np.exp(-g * tau), g ** tau, np.sqrt((k * k).sum())
        u = s * v
        G = np.outer(q / 2.0, Wo[0, 0, 0]) + Ws[0, 0]                       # sqrt(dk) = 2
        dkh, da = G @ u, (G * S0).sum(1)
        dkk = dkh * w / n - (0 if drop_norm_term else k * (dkh * w * k).sum() / n ** 3)
        dw = 0 if forget_alpha_hat else dkh * k / n
        sign = 1.0 if wrong_decay_sign else -1.0
        dg = sign * da * al * tau + dw * tau * g ** (tau - 1)
        return dkk, dg / (1 + np.exp(-zg))

    dkk, dzg = by_hand()
    np.testing.assert_allclose(good["dk"][0, 0, 0], dkk, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(good["dz_g"][0, 0, 0], dzg, rtol=1e-10, atol=1e-12)
    for mistake in ("drop_norm_term", "wrong_decay_sign", "forget_alpha_hat"):
        dkk_bad, dzg_bad = by_hand(**{mistake: True})
        worst = max(np.abs(dkk_bad - dkk).max() / np.abs(dkk).max(), np.abs(dzg_bad - dzg).max() / np.abs(dzg).max())
        assert worst > 1e-2, mistake
