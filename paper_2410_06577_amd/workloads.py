"""Seeded synthetic inputs for the Rodimus DDTS recurrence (no method arithmetic here).

This module only DRAWS inputs; it evaluates neither the recurrence nor any part
of it.  Tests, the smoke check and the benchmark feed the same arrays to the GPU
library and to the CPU oracle.  It depends on numpy and torch (CPU) only and
imports neither the HIP binding nor the oracle.

Recipe (shapes follow the paper's 1.3B/1.6B-class layer: model width 2048, value
width m = 2d = 4096 split over 16 heads, key width n = 64 per head):

    draw order, one numpy PCG64 stream per seed:  q, k, v, z_g, tau, z_beta, S0
    q, k, v   ~ N(0, 1) in fp32;  k <- k / ||k||_2 over dk (the block normalises k)
    log_alpha = -softplus(z_g) * tau,  z_g ~ N(gate_mean, 1),  tau ~ U(tau_lo, tau_hi)
                (the decay gate of the paper, Sec. 3.1.2: alpha = exp(-g .* tau))
    beta      = sigmoid(z_beta),  z_beta ~ N(0, 1)      (the value input gate)
    S0        ~ N(0, s0_std) in fp32, or absent
    q, k, v are then rounded to bf16 (round-to-nearest-even) when io_dtype is bf16.
"""
from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class ScanWorkload:
    name: str
    B: int
    T: int
    H: int
    dk: int
    dv: int
    chunk: int
    io_dtype: str = "bf16"            # "bf16" or "f32": dtype of q, k, v, o
    gate_mean: float = 0.0            # mean of the pre-activation of the decay gate
    tau_range: Optional[Tuple[float, float]] = (0.5, 1.0)   # None: tau == 1
    s0_std: float = 0.0               # 0: no initial state
    seed: int = 0

    @property
    def tokens(self) -> int:
        return self.B * self.T

    @property
    def token_heads(self) -> int:
        return self.B * self.T * self.H


@dataclass(frozen=True)
class DecodeWorkload:
    name: str
    N: int
    H: int
    dk: int
    dv: int
    steps: int
    ring: int = 8                     # distinct token vectors cycled through the chained steps
    io_dtype: str = "bf16"
    s_std: float = 0.1
    seed: int = 4


# The five configurations of the build's baseline file, in its order.
TINY = ScanWorkload("tiny_f32", B=1, T=64, H=1, dk=16, dv=32, chunk=16, io_dtype="f32", seed=0)
MID = ScanWorkload("mid_bf16", B=4, T=2048, H=8, dk=64, dv=128, chunk=64, seed=1)
LAYER_1P6B = ScanWorkload("layer_1p6b", B=8, T=4096, H=16, dk=64, dv=256, chunk=64, s0_std=0.1, seed=2)
LONG_CONTEXT = ScanWorkload("long_context", B=1, T=32768, H=16, dk=64, dv=256, chunk=64,
                            gate_mean=-4.0, tau_range=None, seed=3)
DECODE = DecodeWorkload("decode_256x16", N=256, H=16, dk=64, dv=256, steps=1000, seed=4)

SCAN_WORKLOADS = {w.name: w for w in (TINY, MID, LAYER_1P6B, LONG_CONTEXT)}


def shrink(w: ScanWorkload, **kw) -> ScanWorkload:
    """Same recipe, other sizes (used for oracle-sized parity cases)."""
    return replace(w, **kw)


def _softplus(z):
    return np.logaddexp(np.float32(0.0), z).astype(np.float32)


def _sigmoid(z):
    return (1.0 / (1.0 + np.exp(-z.astype(np.float64)))).astype(np.float32)


def _io(x: np.ndarray, io_dtype: str) -> torch.Tensor:
    t = torch.from_numpy(x)
    if io_dtype == "bf16":
        return t.to(torch.bfloat16)       # round-to-nearest-even
    if io_dtype == "f32":
        return t
    raise ValueError(io_dtype)


def _draw_token_inputs(rng, lead, dk, dv, gate_mean, tau_range, io_dtype):
    f32 = np.float32
    q = rng.standard_normal(lead + (dk,), dtype=f32)
    k = rng.standard_normal(lead + (dk,), dtype=f32)
    v = rng.standard_normal(lead + (dv,), dtype=f32)
    z_g = rng.standard_normal(lead + (dk,), dtype=f32) + f32(gate_mean)
    if tau_range is None:
        tau = np.ones(lead + (dk,), dtype=f32)
    else:
        tau = rng.uniform(tau_range[0], tau_range[1], size=lead + (dk,)).astype(f32)
    z_b = rng.standard_normal(lead + (dv,), dtype=f32)
    k /= np.linalg.norm(k, axis=-1, keepdims=True)
    log_alpha = -(_softplus(z_g) * tau)
    beta = _sigmoid(z_b)
    return {
        "q": _io(q, io_dtype), "k": _io(k, io_dtype), "v": _io(v, io_dtype),
        "log_alpha": torch.from_numpy(log_alpha.astype(f32)),
        "beta": torch.from_numpy(beta),
        "z_beta": _io(z_b, io_dtype),     # the same gate as a pre-activation in the I/O dtype (for the *_zbeta calls)
    }


def make_scan_inputs(w: ScanWorkload) -> dict:
    """CPU tensors q,k,log_alpha [B,T,H,dk]; v,beta,z_beta [B,T,H,dv]; S0 [B,H,dk,dv] fp32 or None."""
    rng = np.random.Generator(np.random.PCG64(w.seed))
    d = _draw_token_inputs(rng, (w.B, w.T, w.H), w.dk, w.dv, w.gate_mean, w.tau_range, w.io_dtype)
    if w.s0_std > 0:
        S0 = rng.standard_normal((w.B, w.H, w.dk, w.dv), dtype=np.float32) * np.float32(w.s0_std)
        d["S0"] = torch.from_numpy(S0)
    else:
        d["S0"] = None
    return d


def make_decode_inputs(w: DecodeWorkload) -> dict:
    """Initial states S [N,H,dk,dv] fp32 and a ring of ``w.ring`` token-vector sets.

    Step i of a chained run uses ring entry i % ring.  Each entry holds
    q,k,log_alpha [N,H,dk] and v,beta [N,H,dv].
    """
    rng = np.random.Generator(np.random.PCG64(w.seed))
    S = rng.standard_normal((w.N, w.H, w.dk, w.dv), dtype=np.float32) * np.float32(w.s_std)
    ring = [_draw_token_inputs(rng, (w.N, w.H), w.dk, w.dv, 0.0, (0.5, 1.0), w.io_dtype)
            for _ in range(w.ring)]
    return {"S": torch.from_numpy(S), "ring": ring}


def make_ddts_preactivations(lead: tuple, dk: int, dv: int, io_dtype: str = "bf16", seed: int = 7) -> dict:
    """Inputs of the DDTS gate front-end: pre-activations z_g, z_tau [lead, dk], z_beta [lead, dv] and raw q, k.

    Drawn so that the resulting gates have the distribution of the scan recipe above: z_g ~ N(0, 1),
    z_tau = logit(U(0.5, 1)) (so that sigmoid(z_tau) ~ U(0.5, 1)), z_beta ~ N(0, 1); q, k ~ N(0, 1), k NOT normalised
    (the front-end normalises it).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    f32 = np.float32
    z_g = rng.standard_normal(lead + (dk,), dtype=f32)
    u = rng.uniform(0.5, 1.0, size=lead + (dk,))
    z_tau = np.log(u / (1.0 - u + 1e-12)).astype(f32)
    z_beta = rng.standard_normal(lead + (dv,), dtype=f32)
    q = rng.standard_normal(lead + (dk,), dtype=f32)
    k = rng.standard_normal(lead + (dk,), dtype=f32)
    return {"z_g": _io(z_g, io_dtype), "z_tau": _io(z_tau, io_dtype), "z_beta": _io(z_beta, io_dtype),
            "q": _io(q, io_dtype), "k": _io(k, io_dtype)}


def serving_length_mix(n_seq: int, total_tokens: int, seed: int = 11) -> list:
    """A prefill batch's length mix: log-uniform lengths (many short prompts, a few long ones), rescaled so that they
    sum to ``total_tokens`` exactly; every sequence has at least one token."""
    rng = np.random.Generator(np.random.PCG64(seed))
    raw = np.exp(rng.uniform(np.log(16.0), np.log(4096.0), size=n_seq))
    lens = np.maximum(1, np.floor(raw * (total_tokens / raw.sum())).astype(np.int64))
    lens[np.argmax(lens)] += total_tokens - lens.sum()
    assert lens.sum() == total_tokens and lens.min() >= 1
    return [int(x) for x in lens]


def make_varlen_inputs(lengths, H: int, dk: int, dv: int, io_dtype: str = "bf16", s0_std: float = 0.1, seed: int = 12) -> dict:
    """Packed variable-length batch: q,k,log_alpha [total,H,dk]; v,beta,z_beta [total,H,dv]; cu_seqlens [N+1] int32;
    S0 [N,H,dk,dv] fp32 or None.  Same per-token recipe as ``make_scan_inputs``."""
    rng = np.random.Generator(np.random.PCG64(seed))
    total = int(sum(lengths))
    d = _draw_token_inputs(rng, (total, H), dk, dv, 0.0, (0.5, 1.0), io_dtype)
    cu = np.zeros(len(lengths) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    d["cu_seqlens"] = torch.from_numpy(cu)
    if s0_std > 0:
        S0 = rng.standard_normal((len(lengths), H, dk, dv), dtype=np.float32) * np.float32(s0_std)
        d["S0"] = torch.from_numpy(S0)
    else:
        d["S0"] = None
    return d


def make_short_conv_inputs(B: int, T: int, C: int, W: int = 4, io_dtype: str = "bf16", seed: int = 13) -> dict:
    """Inputs of the block's ShortConv: x [B,T,C] ~ N(0,1) and a carried history state [B,W-1,C] ~ N(0,1) in the I/O
    dtype; taps w [C,W] and bias [C] in fp32, uniform in +-1/sqrt(W) (the usual initialisation of a depthwise
    convolution of that width)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    f32 = np.float32
    x = rng.standard_normal((B, T, C), dtype=f32)
    state = rng.standard_normal((B, W - 1, C), dtype=f32)
    bound = 1.0 / np.sqrt(W)
    w = rng.uniform(-bound, bound, size=(C, W)).astype(f32)
    bias = rng.uniform(-bound, bound, size=(C,)).astype(f32)
    return {"x": _io(x, io_dtype), "state": _io(state, io_dtype), "w": torch.from_numpy(w), "bias": torch.from_numpy(bias)}


def make_gated_scan_inputs(B: int, T: int, H: int, dk: int, dv: int, io_dtype: str = "bf16", s0_std: float = 0.1,
                           seed: int = 16) -> dict:
    """Inputs of the scan that takes the gates as pre-activations: ``make_ddts_preactivations`` over [B,T,H] plus the
    value v ~ N(0,1) [B,T,H,dv] (I/O dtype) and the initial state S0 ~ N(0, s0_std) fp32 (None when s0_std == 0)."""
    d = make_ddts_preactivations((B, T, H), dk, dv, io_dtype, seed)
    rng = np.random.Generator(np.random.PCG64(seed + 1000))
    d["v"] = _io(rng.standard_normal((B, T, H, dv), dtype=np.float32), io_dtype)
    d["S0"] = torch.from_numpy((rng.standard_normal((B, H, dk, dv), dtype=np.float32) * np.float32(s0_std))) if s0_std > 0 else None
    return d


def make_value_transition_gate(shape: tuple, seed: int = 18, mean: float = -3.0) -> torch.Tensor:
    """log of a transition gate along the value dimension (the beta_t of the general recurrence): -softplus(N(mean, 1)),
    i.e. mostly weak decays (around 0.05 per step for mean = -3) with a tail of stronger ones; fp32, shape [..., dv]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    z = rng.standard_normal(shape, dtype=np.float32) + np.float32(mean)
    return torch.from_numpy((-_softplus(z)).astype(np.float32))
