"""Chunkwise form of the Rodimus recurrence in numpy fp64 -- test infrastructure only.

Follows the appendix "Chunkwise Parallel Representation of the Rodimus Block":
the sequence is cut into consecutive chunks of length C (the paper's B); inside a
chunk the quadratic parallel form gives the intra-chunk output, and a recurrence
over chunks carries the state:

    S_[i]      = diag(prod_{j in chunk i} alpha_j) S_[i-1]
                 + (K_[i] .* Gamma_[i])^T (V_[i] .* beta_[i]),
                 Gamma_[i][b] = prod of alpha over the tokens AFTER row b in the chunk
    O_[i]inter = (Q_[i] .* A_[i]) S_[i-1],
                 A_[i][b] = prod of alpha over rows 1..b of the chunk (row b included)
    O_[i]intra = ((Q .* A)(K / A)^T .* M)(V .* beta)   restricted to the chunk,
                 M lower-triangular INCLUSIVE 0/1
    O_[i]      = O_[i]intra + O_[i]inter

Readings taken where the appendix is loose (all pinned by chunkwise == sequential):
the inter-chunk output uses the state ENTERING the chunk (the printed S_[i] would
count the chunk's own tokens twice); the two outputs are summed; the mask is 0/1 and
includes the diagonal.  The ratio A_t / A_i is evaluated as the product
prod_{j=i+1..t} alpha_j, which is the same number wherever the ratio is defined and
stays defined when some alpha is 0.

This file is a second statement of the method used only to check the chunk algebra
(final state and outputs must not depend on C).  It is not the parity reference;
``sequential.scan`` is.
"""
import numpy as np


def _pairwise_decay(alpha):
    """W[t, i, :] = prod_{j=i+1..t} alpha[j, :] for i <= t, 0 for i > t.  alpha: [C, dk]."""
    C, dk = alpha.shape
    W = np.zeros((C, C, dk), dtype=np.float64)
    for i in range(C):
        W[i, i] = 1.0
        for t in range(i + 1, C):
            W[t, i] = W[t - 1, i] * alpha[t]
    return W


def scan_chunkwise(q, k, v, log_alpha, beta=None, S0=None, chunk=64):
    """Same contract as ``sequential.scan`` (numpy in, float64 out), any chunk >= 1.

    A ragged last chunk (T not a multiple of ``chunk``) is simply shorter.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    la = np.asarray(log_alpha, dtype=np.float64)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    gv = v if beta is None else v * np.asarray(beta, dtype=np.float64)
    alpha = np.exp(la)
    o = np.zeros((B, T, H, dv), dtype=np.float64)
    S_T = np.zeros((B, H, dk, dv), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            S = np.zeros((dk, dv)) if S0 is None else np.asarray(S0[b, h], dtype=np.float64).copy()
            for s in range(0, T, chunk):
                e = min(s + chunk, T)
                Q, K, GV, A = q[b, s:e, h], k[b, s:e, h], gv[b, s:e, h], alpha[b, s:e, h]
                W = _pairwise_decay(A)                      # [C, C, dk]
                cum = W[:, 0, :] * A[0]                     # rows 1..b of the chunk, inclusive
                tail = W[-1, :, :]                          # tokens after row b, to the chunk end
                P = np.einsum("tn,in,tin->ti", Q, K, W)     # masked decayed scores
                o_intra = P @ GV
                o_inter = (Q * cum) @ S
                o[b, s:e, h] = o_intra + o_inter
                S = cum[-1][:, None] * S + (K * tail).T @ GV
            S_T[b, h] = S
    return o, S_T
