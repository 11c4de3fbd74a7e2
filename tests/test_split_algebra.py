"""Host check of the score decomposition the HIP scan kernels use (CPU only, numpy fp64).

The kernels never form the quotient A_t / A_i of the appendix's parallel form.  They build the decayed
scores  P[t,i] = sum_n q_t[n] k_i[n] prod_{j=i+1..t} alpha_j[n]  from products only, by binary splitting:
for each power of two h one array X_h holds, per row, either q .* (prefix product inside the row's h-block)
when bit h of the row index is set, or k .* (suffix product inside the h-block) when it is clear.  The Gram
matrix X_h X_h^T restricted to pairs (t has bit h, i has not, both in the same 2h-block) is exactly the part
of P whose rows split at level h.  This test writes that construction out and compares it with the direct
definition, including alpha = 0 and decays whose quotient form would overflow.
"""
import numpy as np

C, DK = 64, 8
LEVELS = (1, 2, 4, 8, 16, 32)


def _direct_scores(q, k, alpha):
    P = np.zeros((C, C))
    for t in range(C):
        for i in range(t + 1):
            w = np.prod(alpha[i + 1:t + 1], axis=0)
            P[t, i] = np.sum(q[t] * k[i] * w)
    return P


def _block_prefix_suffix(alpha, h):
    """pp[t] = prod of alpha over t's h-block from its start through t; sp[i] = prod over the rows after i."""
    pp, sp = np.ones_like(alpha), np.ones_like(alpha)
    for t in range(C):
        s = t - t % h
        pp[t] = np.prod(alpha[s:t + 1], axis=0)
        sp[t] = np.prod(alpha[t + 1:s + h], axis=0)
    return pp, sp


def _split_scores(q, k, alpha):
    t_idx, i_idx = np.meshgrid(np.arange(C), np.arange(C), indexing="ij")
    P = np.diag(np.sum(q * k, axis=1))                       # a token sees its own write undecayed
    for h in LEVELS:
        pp, sp = _block_prefix_suffix(alpha, h)
        bit = (np.arange(C) & h) != 0
        X = np.where(bit[:, None], q * pp, k * sp)           # one array per level
        gram = X @ X.T
        keep = ((t_idx & h) != 0) & ((i_idx & h) == 0) & (t_idx // (2 * h) == i_idx // (2 * h))
        P = P + np.where(keep, gram, 0.0)
    return P


def _case(seed, resets=False, strong=False):
    rng = np.random.default_rng(seed)
    q, k = rng.standard_normal((C, DK)), rng.standard_normal((C, DK))
    la = -np.abs(rng.standard_normal((C, DK))) * (40.0 if strong else 1.0)
    if resets:
        la[5, :] = -np.inf
        la[33, 2] = -np.inf
        la[48:52, 1] = -np.inf
    return q, k, np.exp(la)


def test_every_pair_belongs_to_exactly_one_level():
    t_idx, i_idx = np.meshgrid(np.arange(C), np.arange(C), indexing="ij")
    count = np.zeros((C, C), int)
    for h in LEVELS:
        count += ((t_idx & h) != 0) & ((i_idx & h) == 0) & (t_idx // (2 * h) == i_idx // (2 * h))
    assert np.array_equal(count, (i_idx < t_idx).astype(int))


def test_split_scores_equal_direct_scores():
    for seed in range(3):
        q, k, alpha = _case(seed)
        np.testing.assert_allclose(_split_scores(q, k, alpha), _direct_scores(q, k, alpha), rtol=1e-12, atol=1e-13)


def test_split_scores_with_resets_and_extreme_decay():
    for kw in (dict(resets=True), dict(strong=True), dict(resets=True, strong=True)):
        q, k, alpha = _case(7, **kw)
        P = _split_scores(q, k, alpha)
        assert np.isfinite(P).all()
        np.testing.assert_allclose(P, _direct_scores(q, k, alpha), rtol=1e-12, atol=1e-13)


def test_level_recurrence_of_the_products():
    """Level 2h follows from level h with one multiply per row (how the kernels build them)."""
    _, _, alpha = _case(3)
    pp, sp = _block_prefix_suffix(alpha, 1)
    for h in LEVELS:
        nxt_pp, nxt_sp = pp.copy(), sp.copy()
        for t in range(C):
            g = t - t % (2 * h)
            if t & h:
                nxt_pp[t] = pp[t] * pp[g + h - 1]            # whole first half, ending at row g+h-1
            else:
                nxt_sp[t] = sp[t] * pp[g + 2 * h - 1]        # whole second half, ending at row g+2h-1
        pp, sp = nxt_pp, nxt_sp
        ref_pp, ref_sp = _block_prefix_suffix(alpha, 2 * h)
        np.testing.assert_allclose(pp, ref_pp, rtol=1e-13)
        np.testing.assert_allclose(sp, ref_sp, rtol=1e-13)
    # after the last level: cumulative decay from the chunk start, and decay to the chunk end
    np.testing.assert_allclose(pp, np.cumprod(alpha, axis=0), rtol=1e-12)
