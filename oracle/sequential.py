"""ctypes front-end of the C oracle (``rodimus_oracle.c``) -- test infrastructure only.

``scan``  : S_t = diag(exp(log_alpha_t)) S_{t-1} + k_t^T (beta_t .* v_t), o_t = q_t S_t
            for t = 1..T (paper Sec. 3.1.3, recurrence of the Rodimus block).
``step``  : one iteration of that recurrence for N independent sequences.

Inputs may be numpy arrays or torch CPU tensors of any float dtype (bf16 included);
they are widened to float32 bit-exactly, the C code widens to double.  Outputs are
numpy float64.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.rodimus_oracle_scan.argtypes = [f32p, f32p, f32p, f32p, f32p, f64p, f64p, f64p] + [ctypes.c_int] * 6
        lib.rodimus_oracle_scan.restype = ctypes.c_int
        lib.rodimus_oracle_step.argtypes = [f32p, f32p, f32p, f32p, f32p, f64p, f64p] + [ctypes.c_int] * 5
        lib.rodimus_oracle_step.restype = ctypes.c_int
        lib.rodimus_oracle_threads.restype = ctypes.c_int
        lib.rodimus_oracle_scan_bwd.argtypes = [f32p] * 5 + [f64p] * 9 + [ctypes.c_int] * 5
        lib.rodimus_oracle_scan_bwd.restype = ctypes.c_int
        lib.rodimus_oracle_scan_bwd_zbeta.argtypes = [f32p] * 5 + [f64p] * 9 + [ctypes.c_int] * 5
        lib.rodimus_oracle_scan_bwd_zbeta.restype = ctypes.c_int
        lib.rodimus_oracle_block_output.argtypes = [f64p, f32p, f32p, f32p, f64p, ctypes.c_long, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.rodimus_oracle_block_output.restype = ctypes.c_int
        lib.rodimus_oracle_scan_gated.argtypes = [f32p] * 6 + [f64p] * 3 + [ctypes.c_int] * 5
        lib.rodimus_oracle_scan_gated.restype = ctypes.c_int
        lib.rodimus_oracle_scan_gated_bwd.argtypes = [f32p] * 6 + [f64p] * 10 + [ctypes.c_int] * 5
        lib.rodimus_oracle_scan_gated_bwd.restype = ctypes.c_int
        lib.rodimus_oracle_step_gated.argtypes = [f32p] * 6 + [f64p] * 2 + [ctypes.c_int] * 4
        lib.rodimus_oracle_step_gated.restype = ctypes.c_int
        lib.rodimus_oracle_scan_general.argtypes = [f32p] * 6 + [f64p] * 3 + [ctypes.c_int] * 5
        lib.rodimus_oracle_scan_general.restype = ctypes.c_int
        lib.rodimus_oracle_step_general.argtypes = [f32p] * 6 + [f64p] * 2 + [ctypes.c_int] * 4
        lib.rodimus_oracle_step_general.restype = ctypes.c_int
        lib.rodimus_oracle_short_conv.argtypes = [f32p, f32p, f32p, f32p, f64p, f64p] + [ctypes.c_int] * 5
        lib.rodimus_oracle_short_conv.restype = ctypes.c_int
        lib.rodimus_oracle_ddts_gates.argtypes = [f32p] * 5 + [f64p] * 4 + [ctypes.c_long, ctypes.c_int, ctypes.c_int]
        lib.rodimus_oracle_ddts_gates.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f32(x):
    """Exact float32 view of a bf16/fp16/fp32 array or tensor (None passes through)."""
    if x is None:
        return None
    if hasattr(x, "detach"):                      # torch tensor, possibly bf16
        x = x.detach().cpu().float().numpy()
    x = np.asarray(x)
    if x.dtype == np.float64:
        y = x.astype(np.float32)
        if not np.array_equal(y.astype(np.float64), x, equal_nan=True):
            raise ValueError("oracle inputs must be exactly representable in float32")
        x = y
    return np.ascontiguousarray(x, dtype=np.float32)


def _f64(x):
    if x is None:
        return None
    if hasattr(x, "detach"):
        x = x.detach().cpu().double().numpy()
    return np.ascontiguousarray(np.asarray(x), dtype=np.float64)


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype)) if a is not None else None


def threads() -> int:
    """Number of host threads the C oracle will use (OpenMP)."""
    return int(_load().rodimus_oracle_threads())


def _value_gate(beta, z_beta):
    if beta is not None and z_beta is not None:
        raise ValueError("give the value gate either as beta or as its pre-activation z_beta, not both")
    return (_f32(z_beta), 1) if z_beta is not None else (_f32(beta), 0)


def scan(q, k, v, log_alpha, beta=None, S0=None, want_state=True, z_beta=None):
    """Sequential oracle.  q,k,log_alpha [B,T,H,dk]; v,beta [B,T,H,dv]; S0 [B,H,dk,dv].

    ``z_beta`` (instead of ``beta``): the value gate's pre-activation, beta = sigmoid(z_beta) (Sec. 3.1.2).
    Returns (o [B,T,H,dv] float64, S_T [B,H,dk,dv] float64 or None).
    """
    lib = _load()
    beta, preact = _value_gate(beta, z_beta)
    q, k, v, la = _f32(q), _f32(k), _f32(v), _f32(log_alpha)
    S0 = _f64(S0)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == (B, T, H, dk) and la.shape == (B, T, H, dk), (k.shape, la.shape)
    assert v.shape == (B, T, H, dv), v.shape
    assert beta is None or beta.shape == (B, T, H, dv), beta.shape
    assert S0 is None or S0.shape == (B, H, dk, dv), S0.shape
    o = np.empty((B, T, H, dv), dtype=np.float64)
    S_T = np.empty((B, H, dk, dv), dtype=np.float64) if want_state else None
    rc = lib.rodimus_oracle_scan(_ptr(q, ctypes.c_float), _ptr(k, ctypes.c_float), _ptr(v, ctypes.c_float),
                                 _ptr(la, ctypes.c_float), _ptr(beta, ctypes.c_float), _ptr(S0, ctypes.c_double),
                                 _ptr(o, ctypes.c_double), _ptr(S_T, ctypes.c_double), B, T, H, dk, dv, preact)
    if rc != 0:
        raise RuntimeError(f"rodimus_oracle_scan failed with code {rc}")
    return o, S_T


def scan_bwd(q, k, v, log_alpha, beta, S0, d_o, dS_T=None, z_beta=None):
    """Backward of ``scan``: cotangents d_o [B,T,H,dv] (and dS_T [B,H,dk,dv] or None) -> dict of float64 gradients
    dq, dk, dlog_alpha [B,T,H,dk]; dv, dbeta (None without beta) [B,T,H,dv]; dS0 [B,H,dk,dv].

    ``z_beta`` (instead of ``beta``): the value gate's pre-activation as in ``scan``; the dict then holds ``dz_beta`` (the
    cotangent of the pre-activation) instead of ``dbeta``."""
    if z_beta is not None:
        if beta is not None:
            raise ValueError("give the value gate either as beta or as its pre-activation z_beta, not both")
        return _scan_bwd_zbeta(q, k, v, log_alpha, z_beta, S0, d_o, dS_T)
    lib = _load()
    q, k, v, la, beta = _f32(q), _f32(k), _f32(v), _f32(log_alpha), _f32(beta)
    S0, d_o, dS_T = _f64(S0), _f64(d_o), _f64(dS_T)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    assert d_o.shape == (B, T, H, dv) and (dS_T is None or dS_T.shape == (B, H, dk, dv))
    out = {"dq": np.zeros((B, T, H, dk)), "dk": np.zeros((B, T, H, dk)), "dlog_alpha": np.zeros((B, T, H, dk)),
           "dv": np.zeros((B, T, H, dv)), "dbeta": None if beta is None else np.zeros((B, T, H, dv)),
           "dS0": np.zeros((B, H, dk, dv))}
    d = ctypes.c_double
    rc = lib.rodimus_oracle_scan_bwd(_ptr(q, ctypes.c_float), _ptr(k, ctypes.c_float), _ptr(v, ctypes.c_float),
                                     _ptr(la, ctypes.c_float), _ptr(beta, ctypes.c_float), _ptr(S0, d), _ptr(d_o, d),
                                     _ptr(dS_T, d), _ptr(out["dq"], d), _ptr(out["dk"], d), _ptr(out["dv"], d),
                                     _ptr(out["dlog_alpha"], d), _ptr(out["dbeta"], d), _ptr(out["dS0"], d), B, T, H, dk, dv)
    if rc != 0:
        raise RuntimeError(f"rodimus_oracle_scan_bwd failed with code {rc}")
    return out


def _scan_bwd_zbeta(q, k, v, log_alpha, z_beta, S0, d_o, dS_T):
    lib = _load()
    q, k, v, la, z_beta = _f32(q), _f32(k), _f32(v), _f32(log_alpha), _f32(z_beta)
    S0, d_o, dS_T = _f64(S0), _f64(d_o), _f64(dS_T)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    assert z_beta.shape == (B, T, H, dv) and d_o.shape == (B, T, H, dv) and (dS_T is None or dS_T.shape == (B, H, dk, dv))
    out = {"dq": np.zeros((B, T, H, dk)), "dk": np.zeros((B, T, H, dk)), "dlog_alpha": np.zeros((B, T, H, dk)),
           "dv": np.zeros((B, T, H, dv)), "dz_beta": np.zeros((B, T, H, dv)), "dS0": np.zeros((B, H, dk, dv))}
    d = ctypes.c_double
    rc = lib.rodimus_oracle_scan_bwd_zbeta(_ptr(q, ctypes.c_float), _ptr(k, ctypes.c_float), _ptr(v, ctypes.c_float),
                                           _ptr(la, ctypes.c_float), _ptr(z_beta, ctypes.c_float), _ptr(S0, d), _ptr(d_o, d),
                                           _ptr(dS_T, d), _ptr(out["dq"], d), _ptr(out["dk"], d), _ptr(out["dv"], d),
                                           _ptr(out["dlog_alpha"], d), _ptr(out["dz_beta"], d), _ptr(out["dS0"], d), B, T, H, dk, dv)
    if rc != 0:
        raise RuntimeError(f"rodimus_oracle_scan_bwd_zbeta failed with code {rc}")
    return out


def block_output(o, x_prime=None, d=None, z_gate=None, act="sigmoid"):
    """Output stage around the recurrence (Sec. 3.1.3): y = (o + d .* x') .* act(z), act in {"sigmoid", "silu"}.

    o [..., H, dv] float64 (a recurrence output); x_prime, z_gate same shape (float32-exact) or None; d [H, dv]."""
    lib = _load()
    o = _f64(o)
    H, dv = o.shape[-2], o.shape[-1]
    rows = o.size // (H * dv)
    x_prime, d, z_gate = _f32(x_prime), _f32(d), _f32(z_gate)
    assert x_prime is None or x_prime.shape == o.shape
    assert z_gate is None or z_gate.shape == o.shape
    assert d is None or d.shape == (H, dv)
    y = np.empty(o.shape, np.float64)
    rc = lib.rodimus_oracle_block_output(_ptr(o, ctypes.c_double), _ptr(x_prime, ctypes.c_float), _ptr(d, ctypes.c_float),
                                         _ptr(z_gate, ctypes.c_float), _ptr(y, ctypes.c_double), rows, H, dv,
                                         {"sigmoid": 0, "silu": 1}[act])
    if rc != 0:
        raise RuntimeError(f"rodimus_oracle_block_output failed with code {rc}")
    return y


def short_conv(x, w, bias=None, state=None, act="silu"):
    """ShortConv (Sec. 3.1.3): causal depthwise convolution over time, width W, then act in {"none", "silu"}.

    x [B, T, C]; w [C, W]; bias [C] or None; state [B, W-1, C] (the previous call's last inputs, oldest first) or None.
    Returns (y [B, T, C], state_out [B, W-1, C]) in float64."""
    lib = _load()
    x, w, bias, state = _f32(x), _f32(w), _f32(bias), _f32(state)
    B, T, C = x.shape
    W = w.shape[1]
    assert w.shape == (C, W)
    assert bias is None or bias.shape == (C,)
    assert state is None or state.shape == (B, W - 1, C)
    y = np.empty((B, T, C), np.float64)
    state_out = np.empty((B, W - 1, C), np.float64)
    rc = lib.rodimus_oracle_short_conv(_ptr(x, ctypes.c_float), _ptr(w, ctypes.c_float), _ptr(bias, ctypes.c_float),
                                       _ptr(state, ctypes.c_float), _ptr(y, ctypes.c_double), _ptr(state_out, ctypes.c_double),
                                       B, T, C, W, {"none": 0, "silu": 1}[act])
    if rc != 0:
        raise RuntimeError(f"rodimus_oracle_short_conv failed with code {rc}")
    return y, state_out


def step(q, k, v, log_alpha, beta, S, z_beta=None):
    """One decode step.  q,k,log_alpha [N,H,dk]; v,beta [N,H,dv]; S [N,H,dk,dv] float64.

    ``z_beta`` as in ``scan``.  Returns (o [N,H,dv] float64, S' float64).  ``S`` itself is not modified.
    """
    lib = _load()
    beta, preact = _value_gate(beta, z_beta)
    q, k, v, la = _f32(q), _f32(k), _f32(v), _f32(log_alpha)
    S = _f64(S).copy()
    N, H, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == (N, H, dk) and la.shape == (N, H, dk)
    assert v.shape == (N, H, dv) and (beta is None or beta.shape == (N, H, dv))
    assert S.shape == (N, H, dk, dv), S.shape
    o = np.empty((N, H, dv), dtype=np.float64)
    rc = lib.rodimus_oracle_step(_ptr(q, ctypes.c_float), _ptr(k, ctypes.c_float), _ptr(v, ctypes.c_float),
                                 _ptr(la, ctypes.c_float), _ptr(beta, ctypes.c_float),
                                 _ptr(S, ctypes.c_double), _ptr(o, ctypes.c_double), N, H, dk, dv, preact)
    if rc != 0:
        raise RuntimeError(f"rodimus_oracle_step failed with code {rc}")
    return o, S


def scan_gated(q, k, v, z_g, z_tau, z_beta=None, S0=None, want_state=True):
    """The block's recurrence from raw q, k and the gates' pre-activations (Sec. 3.1.3 with the gates of Sec. 3.1.2):
    decay exp(-softplus(z_g) sigmoid(z_tau)), key write softplus(z_g)^sigmoid(z_tau) .* k / ||k||, value gate
    sigmoid(z_beta) (None: 1), query q / sqrt(dk).  Shapes as ``scan``.  Returns (o, S_T) float64."""
    lib = _load()
    q, k, v, z_g, z_tau, z_beta = _f32(q), _f32(k), _f32(v), _f32(z_g), _f32(z_tau), _f32(z_beta)
    S0 = _f64(S0)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == z_g.shape == z_tau.shape == (B, T, H, dk) and v.shape == (B, T, H, dv)
    assert z_beta is None or z_beta.shape == (B, T, H, dv)
    assert S0 is None or S0.shape == (B, H, dk, dv)
    o = np.empty((B, T, H, dv), dtype=np.float64)
    S_T = np.empty((B, H, dk, dv), dtype=np.float64) if want_state else None
    f = ctypes.c_float
    rc = lib.rodimus_oracle_scan_gated(_ptr(q, f), _ptr(k, f), _ptr(v, f), _ptr(z_g, f), _ptr(z_tau, f), _ptr(z_beta, f),
                                       _ptr(S0, ctypes.c_double), _ptr(o, ctypes.c_double), _ptr(S_T, ctypes.c_double),
                                       B, T, H, dk, dv)
    if rc != 0:
        raise RuntimeError(f"rodimus_oracle_scan_gated failed with code {rc}")
    return o, S_T


def scan_gated_bwd(q, k, v, z_g, z_tau, z_beta, S0, d_o, dS_T=None):
    """Backward pass of ``scan_gated``: cotangents of the raw q, k, v, of the three pre-activations and of S0, from d_o
    (cotangent of the outputs) and dS_T (of the final state, None = zero).  Returns a dict of float64 arrays ``dq, dk, dv,
    dz_g, dz_tau, dz_beta, dS0`` (``dz_beta`` is None without a value gate)."""
    lib = _load()
    q, k, v, z_g, z_tau, z_beta = _f32(q), _f32(k), _f32(v), _f32(z_g), _f32(z_tau), _f32(z_beta)
    S0, d_o, dS_T = _f64(S0), _f64(d_o), _f64(dS_T)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == z_g.shape == z_tau.shape == (B, T, H, dk) and v.shape == d_o.shape == (B, T, H, dv)
    assert z_beta is None or z_beta.shape == (B, T, H, dv)
    assert S0 is None or S0.shape == (B, H, dk, dv)
    assert dS_T is None or dS_T.shape == (B, H, dk, dv)
    out = {"dq": np.zeros((B, T, H, dk)), "dk": np.zeros((B, T, H, dk)), "dv": np.zeros((B, T, H, dv)),
           "dz_g": np.zeros((B, T, H, dk)), "dz_tau": np.zeros((B, T, H, dk)),
           "dz_beta": np.zeros((B, T, H, dv)) if z_beta is not None else None, "dS0": np.zeros((B, H, dk, dv))}
    f, d = ctypes.c_float, ctypes.c_double
    rc = lib.rodimus_oracle_scan_gated_bwd(_ptr(q, f), _ptr(k, f), _ptr(v, f), _ptr(z_g, f), _ptr(z_tau, f), _ptr(z_beta, f),
                                           _ptr(S0, d), _ptr(d_o, d), _ptr(dS_T, d), _ptr(out["dq"], d), _ptr(out["dk"], d),
                                           _ptr(out["dv"], d), _ptr(out["dz_g"], d), _ptr(out["dz_tau"], d), _ptr(out["dz_beta"], d),
                                           _ptr(out["dS0"], d), B, T, H, dk, dv)
    if rc != 0:
        raise RuntimeError(f"rodimus_oracle_scan_gated_bwd failed with code {rc}")
    return out


def step_gated(q, k, v, z_g, z_tau, z_beta, S):
    """One decode step of ``scan_gated``.  [N,H,.] inputs, S [N,H,dk,dv] float64 (not modified).  Returns (o, S')."""
    lib = _load()
    q, k, v, z_g, z_tau, z_beta = _f32(q), _f32(k), _f32(v), _f32(z_g), _f32(z_tau), _f32(z_beta)
    S = _f64(S).copy()
    N, H, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == z_g.shape == z_tau.shape == (N, H, dk) and v.shape == (N, H, dv) and S.shape == (N, H, dk, dv)
    o = np.empty((N, H, dv), dtype=np.float64)
    f = ctypes.c_float
    rc = lib.rodimus_oracle_step_gated(_ptr(q, f), _ptr(k, f), _ptr(v, f), _ptr(z_g, f), _ptr(z_tau, f), _ptr(z_beta, f),
                                       _ptr(S, ctypes.c_double), _ptr(o, ctypes.c_double), N, H, dk, dv)
    if rc != 0:
        raise RuntimeError(f"rodimus_oracle_step_gated failed with code {rc}")
    return o, S


def scan_general(q, k, v, log_alpha, log_beta_t, beta=None, S0=None, want_state=True):
    """The recurrence with the general transition of Sec. 3.1.1: S_t = (alpha_t^T beta_t) .* S_{t-1} + k_t^T (beta_hat_t .* v_t),
    beta_t = exp(log_beta_t) [B,T,H,dv]; ``beta`` is the input gate beta_hat as in ``scan``.  Returns (o, S_T) float64."""
    lib = _load()
    q, k, v, la, lb, beta = _f32(q), _f32(k), _f32(v), _f32(log_alpha), _f32(log_beta_t), _f32(beta)
    S0 = _f64(S0)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == la.shape == (B, T, H, dk) and v.shape == lb.shape == (B, T, H, dv)
    assert beta is None or beta.shape == (B, T, H, dv)
    o = np.empty((B, T, H, dv), dtype=np.float64)
    S_T = np.empty((B, H, dk, dv), dtype=np.float64) if want_state else None
    f = ctypes.c_float
    rc = lib.rodimus_oracle_scan_general(_ptr(q, f), _ptr(k, f), _ptr(v, f), _ptr(la, f), _ptr(lb, f), _ptr(beta, f),
                                         _ptr(S0, ctypes.c_double), _ptr(o, ctypes.c_double), _ptr(S_T, ctypes.c_double),
                                         B, T, H, dk, dv)
    if rc != 0:
        raise RuntimeError(f"rodimus_oracle_scan_general failed with code {rc}")
    return o, S_T


def step_general(q, k, v, log_alpha, log_beta_t, beta, S):
    """One decode step of ``scan_general``.  Returns (o, S'); ``S`` is not modified."""
    lib = _load()
    q, k, v, la, lb, beta = _f32(q), _f32(k), _f32(v), _f32(log_alpha), _f32(log_beta_t), _f32(beta)
    S = _f64(S).copy()
    N, H, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == la.shape == (N, H, dk) and v.shape == lb.shape == (N, H, dv) and S.shape == (N, H, dk, dv)
    o = np.empty((N, H, dv), dtype=np.float64)
    f = ctypes.c_float
    rc = lib.rodimus_oracle_step_general(_ptr(q, f), _ptr(k, f), _ptr(v, f), _ptr(la, f), _ptr(lb, f), _ptr(beta, f),
                                         _ptr(S, ctypes.c_double), _ptr(o, ctypes.c_double), N, H, dk, dv)
    if rc != 0:
        raise RuntimeError(f"rodimus_oracle_step_general failed with code {rc}")
    return o, S


def ddts_gates(z_g, z_tau, z_beta, q, k):
    """DDTS gate front-end (paper Sec. 3.1.2 and the pre-processing of Sec. 3.1.3), any leading shape [..., dk] / [..., dv].

    Returns float64 arrays (log_alpha, beta or None, q_out, k_out):
    log_alpha = -softplus(z_g) * sigmoid(z_tau), beta = sigmoid(z_beta), q_out = q / sqrt(dk),
    k_out = softplus(z_g)**sigmoid(z_tau) * k / max(||k||_2, 1e-12).
    """
    lib = _load()
    z_g, z_tau, z_beta, q, k = _f32(z_g), _f32(z_tau), _f32(z_beta), _f32(q), _f32(k)
    dk = q.shape[-1]
    M = q.size // dk
    dv = 0 if z_beta is None else z_beta.shape[-1]
    assert z_g.shape == q.shape == k.shape == z_tau.shape
    assert z_beta is None or z_beta.size == M * dv
    la = np.empty(q.shape, np.float64)
    qo = np.empty(q.shape, np.float64)
    ko = np.empty(q.shape, np.float64)
    beta = None if z_beta is None else np.empty(z_beta.shape, np.float64)
    rc = lib.rodimus_oracle_ddts_gates(_ptr(z_g, ctypes.c_float), _ptr(z_tau, ctypes.c_float), _ptr(z_beta, ctypes.c_float),
                                       _ptr(q, ctypes.c_float), _ptr(k, ctypes.c_float), _ptr(la, ctypes.c_double),
                                       _ptr(beta, ctypes.c_double), _ptr(qo, ctypes.c_double), _ptr(ko, ctypes.c_double),
                                       M, dk, dv)
    if rc != 0:
        raise RuntimeError(f"rodimus_oracle_ddts_gates failed with code {rc}")
    return la, beta, qo, ko
