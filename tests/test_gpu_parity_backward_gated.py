"""GPU parity of rodimus_chunk_scan_bwd_gated (the backward pass of the gated scan, through the DDTS gates, the key
normalisation and the query scaling) against the fp64 oracle ``scan_gated_bwd`` (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, rel_err, to_dev

pytestmark = pytest.mark.gpu

NAMES = ("dq", "dk", "dv", "dz_g", "dz_tau", "dz_beta", "dS0")


def _check(B, T, H, dv, seed, with_beta=True, with_dS=True, mutate=None, label=""):
    d = wl.make_gated_scan_inputs(B, T, H, 64, dv, "bf16", seed=seed)
    if not with_beta:
        d["z_beta"] = None
    if mutate is not None:
        mutate(d)
    gen = torch.Generator().manual_seed(seed + 1)
    d_o = torch.randn((B, T, H, dv), generator=gen).to(torch.bfloat16)
    dS_T = (0.1 * torch.randn((B, H, 64, dv), generator=gen)) if with_dS else None
    g = to_dev(d)
    out = rodimus.rodimus_chunk_scan_bwd_gated(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["z_beta"], g["S0"], d_o.cuda(),
                                               None if dS_T is None else dS_T.cuda())
    torch.cuda.synchronize()
    ref = oracle.scan_gated_bwd(d["q"], d["k"], d["v"], d["z_g"], d["z_tau"], d["z_beta"], d["S0"], d_o, dS_T)
    errs = {}
    for name in NAMES:
        if ref[name] is None:
            assert out[name] is None
            continue
        errs[name] = rel_err(out[name], ref[name])
    print(f"   {label} " + " ".join(f"{k} {v:.2e}" for k, v in errs.items()), flush=True)
    for name, e in errs.items():
        assert e <= TOL_BF16, (label, name, e)
    return errs


@pytest.mark.parametrize("B,T,H,dv", [(1, 64, 1, 128), (2, 200, 2, 256), (1, 333, 3, 128)])
def test_small_shapes(B, T, H, dv):
    print(f"gated backward B{B} T{T} H{H} dv{dv}", flush=True)
    _check(B, T, H, dv, seed=T, label="small")


def test_without_value_gate_and_final_state_cotangent():
    _check(1, 150, 2, 256, seed=3, with_beta=False, with_dS=False, label="no z_beta, no dS_T")


def test_zero_and_tiny_keys_take_the_norm_guard():
    def mutate(d):
        d["k"][0, 10, 0] = 0.0                                         # nothing written, gradient through the guard only
        d["k"][0, 40:44, 1] = (d["k"][0, 40:44, 1].float() * 1e-16).to(torch.bfloat16)      # norms below 1e-12
    errs = _check(1, 100, 2, 128, seed=8, mutate=mutate, label="guard")
    assert np.isfinite(list(errs.values())).all()


def test_whole_sequences_at_layer_head_shape():
    # enough (batch, head) pairs that the call is not cut: the sweeps evaluate the gates themselves while they stage a tile
    print("gated backward, uncut, layer head shape", flush=True)
    _check(6, 1024, 16, 256, seed=22, label="uncut")


def test_layer_head_shape_full_length():
    # one sequence of the 1.6B-class layer: T = 4096, 16 heads of 64 x 256 (the call is cut along the sequence)
    print("gated backward layer head shape", flush=True)
    _check(1, 4096, 16, 256, seed=21, label="layer")
