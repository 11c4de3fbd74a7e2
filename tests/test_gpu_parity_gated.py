"""GPU parity of the calls that take every gate as its pre-activation (rodimus_chunk_scan_fwd_gated,
rodimus_decode_step_gated) against the fp64 oracle of the block's recurrence (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, TOL_F32, rel_err, to_dev

pytestmark = pytest.mark.gpu


def _check_scan(d, chunk, tol, use_zbeta=True, label=""):
    g = to_dev(d)
    o, S_T = rodimus.rodimus_chunk_scan_fwd_gated(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"],
                                                  g["z_beta"] if use_zbeta else None, g["S0"], chunk=chunk)
    torch.cuda.synchronize()
    o_ref, S_ref = oracle.scan_gated(d["q"], d["k"], d["v"], d["z_g"], d["z_tau"], d["z_beta"] if use_zbeta else None, d["S0"])
    eo, es = rel_err(o, o_ref), rel_err(S_T, S_ref)
    assert eo <= tol and es <= tol, f"{label}: o {eo:.3e} S_T {es:.3e} > {tol}"
    return o, S_T


@pytest.mark.parametrize("B,T,H,dk,dv,chunk,io", [
    (2, 300, 3, 64, 256, 64, "bf16"),      # matrix-core kernel, ragged tail
    (1, 130, 2, 64, 128, 64, "bf16"),
    (1, 2048, 2, 64, 256, 64, "bf16"),     # few workgroups: the sequence-split path (summary pass with the gates fused)
    (2, 50, 2, 16, 32, 16, "f32"),         # generic kernel
    (1, 77, 3, 32, 40, 32, "bf16"),
    (2, 20, 1, 8, 8, 4, "f32"),
])
def test_gated_scan_matches_the_oracle(B, T, H, dk, dv, chunk, io):
    print(f"gated scan B{B} T{T} H{H} dk{dk} dv{dv} C{chunk} {io}", flush=True)
    d = wl.make_gated_scan_inputs(B, T, H, dk, dv, io, seed=T + dv)
    tol = TOL_BF16 if io == "bf16" else TOL_F32
    _check_scan(d, chunk, tol, True, "with z_beta")
    _check_scan(d, chunk, tol, False, "without value gate")


@pytest.mark.parametrize("dk,dv,chunk,io", [(64, 256, 64, "bf16"), (16, 32, 16, "f32")])
def test_gated_scan_extreme_gates_and_zero_keys(dk, dv, chunk, io):
    B, T, H = 1, 160, 2
    d = wl.make_gated_scan_inputs(B, T, H, dk, dv, io, seed=5)
    d["z_g"][:, 10:14] = 30.0            # g = 30: a near reset inside a tile (the product-only route of the matrix-core kernel)
    d["z_tau"][:, 10:14] = 20.0
    d["z_g"][:, 40:60] = -100.0          # g underflows: no decay, nothing written (g^tau -> 0)
    d["z_tau"][:, 70:75] = -100.0        # tau -> 0: no decay, key gate -> 1
    d["k"][:, 90:93] = 0.0               # zero keys stay zero under the normalisation guard
    d["z_g"][:, 100:104, :, : dk // 2] = 90.0     # half the channels reset hard
    d["z_tau"][:, 100:104, :, : dk // 2] = 90.0
    _check_scan(d, chunk, TOL_BF16 if io == "bf16" else TOL_F32, True, "extremes")


def test_gated_scan_agrees_with_the_two_call_pipeline():
    d = wl.make_gated_scan_inputs(2, 200, 2, 64, 256, "bf16", seed=9)
    g = to_dev(d)
    o1, S1 = rodimus.rodimus_chunk_scan_fwd_gated(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["z_beta"], g["S0"])
    la, _, qo, ko = rodimus.rodimus_ddts_gates(g["z_g"], g["z_tau"], None, g["q"], g["k"])
    o2, S2 = rodimus.rodimus_chunk_scan_fwd_zbeta(qo, ko, g["v"], la, g["z_beta"], g["S0"])
    torch.cuda.synchronize()
    # same arithmetic except the order in which the squared key norm is summed
    assert rel_err(o1, o2.double().cpu().numpy()) <= 1e-2
    assert rel_err(S1, S2.double().cpu().numpy()) <= 1e-3


@pytest.mark.parametrize("N,H,dk,dv,io", [(5, 3, 64, 256, "bf16"), (2, 2, 16, 32, "f32"), (3, 1, 200, 24, "f32"),
                                          (2, 2, 256, 260, "bf16")])
def test_gated_decode_step_matches_the_oracle_and_chains_to_the_scan(N, H, dk, dv, io):
    print(f"gated decode N{N} H{H} dk{dk} dv{dv} {io}", flush=True)
    T = 6
    d = wl.make_gated_scan_inputs(N, T, H, dk, dv, io, seed=dk + dv)
    g = to_dev(d)
    tol = TOL_BF16 if io == "bf16" else TOL_F32
    S = g["S0"].clone()
    S_ref = d["S0"].double().numpy()
    for t in range(T):
        sl = lambda x: x[:, t].contiguous()
        o = rodimus.rodimus_decode_step_gated(sl(g["q"]), sl(g["k"]), sl(g["v"]), sl(g["z_g"]), sl(g["z_tau"]), sl(g["z_beta"]), S)
        torch.cuda.synchronize()
        # every step against the oracle started from the GPU's own state before the step
        o_ref, S_next = oracle.step_gated(d["q"][:, t], d["k"][:, t], d["v"][:, t], d["z_g"][:, t], d["z_tau"][:, t],
                                          d["z_beta"][:, t], S_ref)
        assert rel_err(o, o_ref) <= tol and rel_err(S, S_next) <= TOL_F32
        S_ref = S.double().cpu().numpy()
    if dk <= 128:
        o_scan, S_scan = rodimus.rodimus_chunk_scan_fwd_gated(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["z_beta"], g["S0"],
                                                              chunk=64 if dk == 64 else 4)
        torch.cuda.synchronize()
        assert rel_err(S_scan, S.double().cpu().numpy()) <= tol
    # without a value gate
    S2 = g["S0"].clone()
    sl = lambda x: x[:, 0].contiguous()
    o = rodimus.rodimus_decode_step_gated(sl(g["q"]), sl(g["k"]), sl(g["v"]), sl(g["z_g"]), sl(g["z_tau"]), None, S2)
    torch.cuda.synchronize()
    o_ref, S_next = oracle.step_gated(d["q"][:, 0], d["k"][:, 0], d["v"][:, 0], d["z_g"][:, 0], d["z_tau"][:, 0], None,
                                      d["S0"].double().numpy())
    assert rel_err(o, o_ref) <= tol and rel_err(S2, S_next) <= TOL_F32
