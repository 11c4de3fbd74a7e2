"""Pins for the fp64 CPU oracle (CPU only).

The oracle is checked against things other than itself: values worked by hand
from the recurrence, textbook operators it must reduce to, the unrolled weighted
sum of the paper evaluated by brute force, closed forms, and invariances.  Each
test names the passage of the paper that fixes the expected result.
"""
import os

import numpy as np
import pytest

import oracle
from oracle.chunkwise import scan_chunkwise

RNG = np.random.default_rng(1234)


def _rand_case(B, T, H, dk, dv, with_s0=True, rng=RNG):
    f = np.float32
    q = rng.standard_normal((B, T, H, dk)).astype(f)
    k = rng.standard_normal((B, T, H, dk)).astype(f)
    v = rng.standard_normal((B, T, H, dv)).astype(f)
    la = (-np.abs(rng.standard_normal((B, T, H, dk)))).astype(f)
    beta = rng.uniform(0.1, 1.0, (B, T, H, dv)).astype(f)
    S0 = rng.standard_normal((B, H, dk, dv)).astype(f) if with_s0 else None
    return q, k, v, la, beta, S0


# --------------------------------------------------------------------------- hand-worked
def _read_golden(path):
    rows = {}
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, vals = line.split(":")
            rows[key.strip()] = np.array([float(x) for x in vals.split()])
    return rows


def test_hand_worked_example(golden_dir):
    """Recurrence of the Rodimus block (Sec. 3.1.3), three steps worked by hand."""
    g = _read_golden(os.path.join(golden_dir, "hand_worked_T3.txt"))
    sh = (1, 3, 1, 2)
    la = np.log(g["alpha"]).astype(np.float32).reshape(sh)
    o, S_T = oracle.scan(g["q"].reshape(sh), g["k"].reshape(sh), g["v"].reshape(sh), la, g["beta"].reshape(sh))
    np.testing.assert_allclose(o.reshape(-1), g["o"], rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(S_T.reshape(-1), g["S_T"], rtol=1e-6, atol=1e-6)


# --------------------------------------------------------------------------- textbook reductions
def test_reduces_to_causal_linear_attention():
    """alpha = 1, beta = 1: un-normalised identity-map linear attention (Sec. 2, S_t = S_{t-1} + k^T v)."""
    B, T, H, dk, dv = 2, 37, 3, 5, 7
    q, k, v, _, _, _ = _rand_case(B, T, H, dk, dv, with_s0=False)
    la = np.zeros((B, T, H, dk), np.float32)
    o, S_T = oracle.scan(q, k, v, la, None, None)
    for b in range(B):
        for h in range(H):
            Q, K, V = (x[b, :, h].astype(np.float64) for x in (q, k, v))
            np.testing.assert_allclose(o[b, :, h], np.tril(Q @ K.T) @ V, rtol=1e-12, atol=1e-12)
            np.testing.assert_allclose(S_T[b, h], K.T @ V, rtol=1e-12, atol=1e-12)
    # the same thing as prefix sums of the outer products
    S = np.cumsum(np.einsum("tn,tm->tnm", k[0, :, 0].astype(np.float64), v[0, :, 0].astype(np.float64)), axis=0)
    np.testing.assert_allclose(o[0, :, 0], np.einsum("tn,tnm->tm", q[0, :, 0].astype(np.float64), S), rtol=1e-12)


def test_alpha_zero_keeps_only_current_outer_product():
    """alpha = 0 (log_alpha = -inf): the state is overwritten each step; the token still sees its own write."""
    B, T, H, dk, dv = 1, 9, 2, 4, 6
    q, k, v, _, beta, S0 = _rand_case(B, T, H, dk, dv)
    la = np.full((B, T, H, dk), -np.inf, np.float32)
    o, S_T = oracle.scan(q, k, v, la, beta, S0)
    qk = np.einsum("bthn,bthn->bth", q.astype(np.float64), k.astype(np.float64))
    gv = beta.astype(np.float64) * v.astype(np.float64)
    np.testing.assert_allclose(o, qk[..., None] * gv, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(S_T, np.einsum("bhn,bhm->bhnm", k[:, -1].astype(np.float64), gv[:, -1]), rtol=1e-12)
    assert np.isfinite(o).all()


def test_scalar_constant_decay_geometric_series_and_retention_mask():
    """Constant scalar decay gamma (the RetNet row of the gate table): mask gamma^(t-i), geometric-series state."""
    T, dk, dv, gamma = 25, 3, 4, 0.8125            # gamma is a dyadic rational
    la = np.full((1, T, 1, dk), np.log(gamma), np.float32)
    gam = float(np.exp(np.float64(la.flat[0])))     # the exact decay the oracle sees
    # closed form: q = k = e_1, v = 1  =>  S_t[0, :] = (1 - gam^t) / (1 - gam)
    q = np.zeros((1, T, 1, dk), np.float32); q[..., 0] = 1
    v = np.ones((1, T, 1, dv), np.float32)
    o, S_T = oracle.scan(q, q, v, la)
    t = np.arange(1, T + 1)
    np.testing.assert_allclose(o[0, :, 0, :], ((1 - gam ** t) / (1 - gam))[:, None] * np.ones(dv), rtol=1e-12)
    np.testing.assert_allclose(S_T[0, 0, 0], (1 - gam ** T) / (1 - gam), rtol=1e-12)
    assert np.all(S_T[0, 0, 1:] == 0)
    # decay mask: o = ((Q K^T) .* D) V with D[t, i] = gam^(t - i), i <= t
    qr, kr, vr, _, _, _ = _rand_case(1, T, 1, dk, dv, with_s0=False)
    o2, _ = oracle.scan(qr, kr, vr, la)
    idx = np.arange(T)
    D = np.where(idx[:, None] >= idx[None, :], gam ** (idx[:, None] - idx[None, :]).clip(0), 0.0)
    Q, K, V = (x[0, :, 0].astype(np.float64) for x in (qr, kr, vr))
    np.testing.assert_allclose(o2[0, :, 0], ((Q @ K.T) * D) @ V, rtol=1e-11, atol=1e-12)


def test_selection_gate_special_case():
    """alpha = 1 - sigmoid(g), input gate sigmoid(g) folded into k (the HGRN2 row of the gate table), dk = 1:
    the state is then an exponential moving average with closed-form weights."""
    T, dv = 12, 3
    g = RNG.standard_normal(T)
    sig = 1 / (1 + np.exp(-g))
    la = np.log1p(-sig).astype(np.float32).reshape(1, T, 1, 1)
    a = np.exp(la.astype(np.float64)).reshape(T)
    k = sig.astype(np.float32).reshape(1, T, 1, 1)
    v = RNG.standard_normal((1, T, 1, dv)).astype(np.float32)
    q = np.ones((1, T, 1, 1), np.float32)
    o, _ = oracle.scan(q, k, v, la)
    kk = k.astype(np.float64).reshape(T)
    for t in range(T):
        w = np.array([kk[i] * np.prod(a[i + 1:t + 1]) for i in range(t + 1)])
        np.testing.assert_allclose(o[0, t, 0], w @ v[0, :t + 1, 0].astype(np.float64), rtol=1e-12, atol=1e-14)


# --------------------------------------------------------------------------- brute force
def _unrolled_weighted_sum(q, k, v, la, beta, S0):
    """The unrolled form of Sec. 3.1.1 (value-side decay = 1) plus the carried-in state, by plain loops:
    o_t = sum_{i<=t} [ q_t (prod_{j=i+1..t} alpha_j .* k_i)^T ] (beta_i .* v_i) + (q_t .* prod_{j<=t} alpha_j) S0."""
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    a = np.exp(la.astype(np.float64))
    o = np.zeros((B, T, H, dv))
    for b in range(B):
        for h in range(H):
            for t in range(T):
                acc = np.zeros(dv)
                for i in range(t + 1):
                    w = 0.0
                    for n in range(dk):
                        p = 1.0
                        for j in range(i + 1, t + 1):
                            p *= a[b, j, h, n]
                        w += float(q[b, t, h, n]) * p * float(k[b, i, h, n])
                    acc += w * (beta[b, i, h].astype(np.float64) * v[b, i, h].astype(np.float64))
                if S0 is not None:
                    p = np.prod(a[b, :t + 1, h], axis=0)
                    acc += (q[b, t, h].astype(np.float64) * p) @ S0[b, h].astype(np.float64)
                o[b, t, h] = acc
    return o


def test_brute_force_unrolled_sum():
    B, T, H, dk, dv = 2, 17, 2, 3, 5
    q, k, v, la, beta, S0 = _rand_case(B, T, H, dk, dv)
    o, _ = oracle.scan(q, k, v, la, beta, S0)
    np.testing.assert_allclose(o, _unrolled_weighted_sum(q, k, v, la, beta, S0), rtol=1e-11, atol=1e-12)


def test_value_gate_given_as_pre_activation():
    """Sec. 3.1.2: the value-side input gate is sigmoid(z_beta).  Given z_beta, the oracle must equal the brute-force
    sum with that gate, coincide with an explicit gate where the sigmoid is exact in float (z = 0 -> 1/2), tend to
    the ungated recurrence for large z and to "nothing written" for z = -inf; the decode step follows the scan."""
    B, T, H, dk, dv = 2, 13, 2, 3, 5
    q, k, v, la, _, S0 = _rand_case(B, T, H, dk, dv)
    z = (2.0 * RNG.standard_normal((B, T, H, dv))).astype(np.float32)
    o, S_T = oracle.scan(q, k, v, la, None, S0, z_beta=z)
    gate = 1.0 / (1.0 + np.exp(-z.astype(np.float64)))
    np.testing.assert_allclose(o, _unrolled_weighted_sum(q, k, v, la, gate, S0), rtol=1e-11, atol=1e-12)

    half = np.full((B, T, H, dv), 0.5, np.float32)
    o_a, S_a = oracle.scan(q, k, v, la, None, S0, z_beta=np.zeros_like(z))
    o_b, S_b = oracle.scan(q, k, v, la, half, S0)
    assert np.array_equal(o_a, o_b) and np.array_equal(S_a, S_b)

    o_a, S_a = oracle.scan(q, k, v, la, None, S0, z_beta=np.full_like(z, 60.0))
    o_b, S_b = oracle.scan(q, k, v, la, None, S0)
    np.testing.assert_allclose(o_a, o_b, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(S_a, S_b, rtol=1e-13, atol=1e-13)

    o_a, S_a = oracle.scan(q, k, v, la, None, S0, z_beta=np.full_like(z, -np.inf))
    o_b, S_b = oracle.scan(q, k, np.zeros_like(v), la, None, S0)
    assert np.array_equal(o_a, o_b) and np.array_equal(S_a, S_b)

    with pytest.raises(ValueError):
        oracle.scan(q, k, v, la, half, S0, z_beta=z)

    o1, S1 = oracle.scan(q[:, :1], k[:, :1], v[:, :1], la[:, :1], None, S0, z_beta=z[:, :1])
    od, Sd = oracle.step(q[:, 0], k[:, 0], v[:, 0], la[:, 0], None, S0, z_beta=z[:, 0])
    assert np.array_equal(od, o1[:, 0]) and np.array_equal(Sd, S1)


# --------------------------------------------------------------------------- invariances
def test_initial_state_only_and_linearity():
    B, T, H, dk, dv = 1, 11, 2, 4, 3
    q, k, v, la, beta, S0 = _rand_case(B, T, H, dk, dv)
    zero_k = np.zeros_like(k)
    o, S_T = oracle.scan(q, zero_k, v, la, beta, S0)
    cum = np.exp(np.cumsum(la.astype(np.float64), axis=1))           # prod_{j<=t} alpha_j
    np.testing.assert_allclose(o, np.einsum("bthn,bhnm->bthm", q * cum, S0.astype(np.float64)), rtol=1e-11)
    np.testing.assert_allclose(S_T, cum[:, -1][..., None] * S0, rtol=1e-11)
    # superposition: (inputs with S0) = (inputs with zero state) + (state alone)
    o_full, S_full = oracle.scan(q, k, v, la, beta, S0)
    o_in, S_in = oracle.scan(q, k, v, la, beta, None)
    np.testing.assert_allclose(o_full, o_in + o, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(S_full, S_in + S_T, rtol=1e-10, atol=1e-12)
    # linear in v
    o2, _ = oracle.scan(q, k, (2 * v).astype(np.float32), la, beta, None)
    np.testing.assert_allclose(o2, 2 * o_in, rtol=1e-12)


def test_split_sequence_resume():
    """The state is the whole memory: scan(0..T) == scan(0..T1) then scan(T1..T) started from S_T1."""
    B, T, H, dk, dv, T1 = 2, 29, 2, 4, 5, 13
    q, k, v, la, beta, S0 = _rand_case(B, T, H, dk, dv)
    o, S_T = oracle.scan(q, k, v, la, beta, S0)
    o1, S1 = oracle.scan(q[:, :T1], k[:, :T1], v[:, :T1], la[:, :T1], beta[:, :T1], S0)
    o2, S2 = oracle.scan(q[:, T1:], k[:, T1:], v[:, T1:], la[:, T1:], beta[:, T1:], S1)
    np.testing.assert_array_equal(np.concatenate([o1, o2], axis=1), o)
    np.testing.assert_array_equal(S2, S_T)


def test_decode_step_is_one_iteration_and_chains_to_scan():
    B, T, H, dk, dv = 3, 7, 2, 4, 6
    q, k, v, la, beta, S0 = _rand_case(B, T, H, dk, dv)
    o, S_T = oracle.scan(q, k, v, la, beta, S0)
    S = S0.astype(np.float64)
    for t in range(T):
        o_t, S = oracle.step(q[:, t], k[:, t], v[:, t], la[:, t], beta[:, t], S)
        np.testing.assert_array_equal(o_t, o[:, t])
    np.testing.assert_array_equal(S, S_T)


def test_layout_heads_and_batches_are_independent():
    """Every (b, h) recurrence only reads its own slices of the [B,T,H,*] arrays."""
    B, T, H, dk, dv = 2, 8, 3, 4, 5
    q, k, v, la, beta, S0 = _rand_case(B, T, H, dk, dv)
    o, S_T = oracle.scan(q, k, v, la, beta, S0)
    for b in range(B):
        for h in range(H):
            sl = lambda x: np.ascontiguousarray(x[b:b + 1, :, h:h + 1])
            o1, S1 = oracle.scan(sl(q), sl(k), sl(v), sl(la), sl(beta), np.ascontiguousarray(S0[b:b + 1, h:h + 1]))
            np.testing.assert_array_equal(o1[0, :, 0], o[b, :, h])
            np.testing.assert_array_equal(S1[0, 0], S_T[b, h])


# --------------------------------------------------------------------------- chunkwise form
@pytest.mark.parametrize("chunk", [1, 2, 16, 64, 80])
def test_chunkwise_form_matches_sequential(chunk):
    """Appendix 'Chunkwise Parallel Representation': outputs and final state do not depend on the chunk size."""
    B, T, H, dk, dv = 1, 80, 2, 6, 5
    q, k, v, la, beta, S0 = _rand_case(B, T, H, dk, dv)
    o, S_T = oracle.scan(q, k, v, la, beta, S0)
    oc, Sc = scan_chunkwise(q, k, v, la, beta, S0, chunk=chunk)
    np.testing.assert_allclose(oc, o, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(Sc, S_T, rtol=1e-10, atol=1e-12)


def test_chunkwise_ragged_tail_and_hard_resets():
    B, T, H, dk, dv = 1, 45, 1, 4, 3
    q, k, v, la, beta, S0 = _rand_case(B, T, H, dk, dv)
    la[0, 7, 0, 1] = -np.inf
    la[0, 20, 0, :] = -np.inf
    o, S_T = oracle.scan(q, k, v, la, beta, S0)
    oc, Sc = scan_chunkwise(q, k, v, la, beta, S0, chunk=16)
    assert np.isfinite(oc).all()
    np.testing.assert_allclose(oc, o, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(Sc, S_T, rtol=1e-10, atol=1e-12)


def test_mutation_sensitivity_of_the_pins():
    """A wrong reading must fail a pin: pre-update output, decayed own write and a transposed state all
    change the hand-worked example (guards against pins that would accept anything)."""
    q = np.array([[1, 1], [1, -1], [2, 1]], float); k = np.array([[1, 2], [1, 0], [0, 1]], float)
    a = np.array([[.5, 1], [.5, .25], [1, .5]]); gv = np.array([[2, 2], [1, -1], [2, 3]], float)
    good = np.array([[6, 6], [1, -1], [6.5, 3.5]])

    def run(variant):
        S = np.zeros((2, 2)); out = []
        for t in range(3):
            if variant == "pre":
                out.append(q[t] @ S)
            w = np.outer(k[t], gv[t])
            if variant == "transposed":
                w = np.outer(gv[t], k[t])
            S = a[t][:, None] * (S + w) if variant == "decay_own" else a[t][:, None] * S + w
            if variant != "pre":
                out.append(q[t] @ S)
        return np.array(out)

    np.testing.assert_allclose(run("good"), good)
    for bad in ("pre", "decay_own", "transposed"):
        assert not np.allclose(run(bad), good), bad


def test_general_transition_unrolled_sum_reduction_and_separable_case():
    """The value-side transition gate of Sec. 3.1.1: the unrolled form printed with it (both gates' products between write
    and read), reduction to the block's recurrence at beta_t = 1, and a closed form where the two gates are constants."""
    rng = np.random.default_rng(31)
    B, T, H, dk, dv = 1, 11, 2, 3, 4
    q = rng.standard_normal((B, T, H, dk)).astype(np.float32)
    k = rng.standard_normal((B, T, H, dk)).astype(np.float32)
    v = rng.standard_normal((B, T, H, dv)).astype(np.float32)
    la = -rng.uniform(0.0, 1.0, (B, T, H, dk)).astype(np.float32)
    lb = -rng.uniform(0.0, 1.0, (B, T, H, dv)).astype(np.float32)
    bh = rng.uniform(0.0, 1.0, (B, T, H, dv)).astype(np.float32)
    o, S_T = oracle.scan_general(q, k, v, la, lb, bh)
    # o_t = sum_{i<=t} [q_t (prod_{j=i+1..t} alpha_j .* k_i)^T] (prod_{j=i+1..t} beta_j .* beta_hat_i .* v_i)
    la64, lb64 = la.astype(np.float64), lb.astype(np.float64)
    for h in range(H):
        for t in range(T):
            acc = np.zeros(dv)
            for i in range(t + 1):
                da = np.exp(la64[0, i + 1:t + 1, h].sum(axis=0))
                db = np.exp(lb64[0, i + 1:t + 1, h].sum(axis=0))
                acc += (q[0, t, h].astype(np.float64) @ (da * k[0, i, h])) * (db * bh[0, i, h].astype(np.float64) * v[0, i, h])
            np.testing.assert_allclose(o[0, t, h], acc, rtol=1e-12, atol=1e-13)
    # beta_t = 1 is the block's recurrence
    zero = np.zeros_like(lb)
    o1, S1 = oracle.scan_general(q, k, v, la, zero, bh)
    o2, S2 = oracle.scan(q, k, v, la, bh)
    assert np.array_equal(o1, o2) and np.array_equal(S1, S2)
    # constant scalar gates a (keys) and b (values): the state decays by (a b)^(t-i): same as the block's recurrence with
    # the key-side gate a * b
    a_log, b_log = np.float32(-0.25), np.float32(-0.5)
    o3, S3 = oracle.scan_general(q, k, v, np.full_like(la, a_log), np.full_like(lb, b_log), None)
    o4, S4 = oracle.scan(q, k, v, np.full_like(la, a_log + b_log), None)
    np.testing.assert_allclose(o3, o4, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(S3, S4, rtol=1e-13, atol=1e-14)
    # decode steps chain to the scan
    S = np.zeros((B, H, dk, dv))
    for t in range(T):
        o_t, S = oracle.step_general(q[:, t], k[:, t], v[:, t], la[:, t], lb[:, t], bh[:, t], S)
        assert np.array_equal(o_t, o[:, t])
    assert np.array_equal(S, S_T)
