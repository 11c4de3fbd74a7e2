"""GPU parity of the general transition of Sec. 3.1.1 (a gate along the value dimension as well):
rodimus_chunk_scan_fwd_general and rodimus_decode_step_general against the fp64 oracle (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, TOL_F32, rel_err, to_dev

pytestmark = pytest.mark.gpu


def _inputs(B, T, H, dk, dv, chunk, io, seed):
    w = wl.ScanWorkload("case", B=B, T=T, H=H, dk=dk, dv=dv, chunk=chunk, io_dtype=io, s0_std=0.1, seed=seed)
    inp = wl.make_scan_inputs(w)
    inp["log_beta_t"] = wl.make_value_transition_gate((B, T, H, dv), seed + 7)
    return inp


@pytest.mark.parametrize("B,T,H,dk,dv,chunk,io", [
    (1, 64, 1, 16, 32, 16, "f32"),
    (2, 100, 2, 32, 72, 32, "f32"),       # two column tiles, the second ragged; ragged last chunk
    (1, 150, 2, 64, 128, 64, "bf16"),     # a shape the matrix-core kernel would take: this form stays on the generic kernel
    (2, 9, 1, 8, 8, 4, "f32"),
])
def test_general_scan_matches_the_oracle(B, T, H, dk, dv, chunk, io):
    print(f"general scan B{B} T{T} H{H} dk{dk} dv{dv} C{chunk} {io}", flush=True)
    inp = _inputs(B, T, H, dk, dv, chunk, io, seed=T + dv)
    g = to_dev(inp)
    tol = TOL_BF16 if io == "bf16" else TOL_F32
    for use_beta in (True, False):
        o, S_T = rodimus.rodimus_chunk_scan_fwd_general(g["q"], g["k"], g["v"], g["log_alpha"], g["log_beta_t"],
                                                        g["beta"] if use_beta else None, g["S0"], chunk=chunk)
        torch.cuda.synchronize()
        o_ref, S_ref = oracle.scan_general(inp["q"], inp["k"], inp["v"], inp["log_alpha"], inp["log_beta_t"],
                                           inp["beta"] if use_beta else None, inp["S0"])
        assert rel_err(o, o_ref) <= tol and rel_err(S_T, S_ref) <= tol


def test_general_scan_strong_and_closed_value_gates_and_chunk_invariance():
    inp = _inputs(1, 96, 2, 16, 32, 16, "f32", seed=3)
    lb = inp["log_beta_t"]
    lb[:, 10:14, :, :8] = -40.0            # a near reset of some columns
    lb[:, 30::17] = float("-inf")          # columns closed outright
    lb[:, 50:60] = 0.0
    g = to_dev(inp)
    o_ref, S_ref = oracle.scan_general(inp["q"], inp["k"], inp["v"], inp["log_alpha"], lb, inp["beta"], inp["S0"])
    outs = []
    for chunk in (16, 5, 64):
        o, S_T = rodimus.rodimus_chunk_scan_fwd_general(g["q"], g["k"], g["v"], g["log_alpha"], g["log_beta_t"], g["beta"],
                                                        g["S0"], chunk=chunk)
        torch.cuda.synchronize()
        assert rel_err(o, o_ref) <= TOL_F32 and rel_err(S_T, S_ref) <= TOL_F32, chunk
        assert torch.isfinite(o).all() and torch.isfinite(S_T).all()
        outs.append(o)
    # with the value gate open everywhere the call is the block's recurrence
    zero = torch.zeros_like(g["log_beta_t"])
    o0, S0 = rodimus.rodimus_chunk_scan_fwd_general(g["q"], g["k"], g["v"], g["log_alpha"], zero, g["beta"], g["S0"], chunk=16)
    o1, S1 = rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], chunk=16)
    torch.cuda.synchronize()
    assert rel_err(o0, o1.double().cpu().numpy()) <= 1e-5 and rel_err(S0, S1.double().cpu().numpy()) <= 1e-5


@pytest.mark.parametrize("N,H,dk,dv,io", [(4, 3, 64, 256, "bf16"), (2, 2, 16, 32, "f32"), (3, 1, 100, 20, "f32")])
def test_general_decode_step_matches_the_oracle_and_chains_to_the_scan(N, H, dk, dv, io):
    print(f"general decode N{N} H{H} dk{dk} dv{dv} {io}", flush=True)
    T = 5
    inp = _inputs(N, T, H, dk, dv, 4, io, seed=dk + dv)
    g = to_dev(inp)
    tol = TOL_BF16 if io == "bf16" else TOL_F32
    S = g["S0"].clone()
    S_ref = inp["S0"].double().numpy()
    for t in range(T):
        sl = lambda x: x[:, t].contiguous()
        o = rodimus.rodimus_decode_step_general(sl(g["q"]), sl(g["k"]), sl(g["v"]), sl(g["log_alpha"]), sl(g["log_beta_t"]),
                                                sl(g["beta"]), S)
        torch.cuda.synchronize()
        o_ref, S_next = oracle.step_general(inp["q"][:, t], inp["k"][:, t], inp["v"][:, t], inp["log_alpha"][:, t],
                                            inp["log_beta_t"][:, t], inp["beta"][:, t], S_ref)
        assert rel_err(o, o_ref) <= tol and rel_err(S, S_next) <= TOL_F32
        S_ref = S.double().cpu().numpy()
    o_scan, S_scan = rodimus.rodimus_chunk_scan_fwd_general(g["q"], g["k"], g["v"], g["log_alpha"], g["log_beta_t"], g["beta"],
                                                            g["S0"], chunk=4)
    torch.cuda.synchronize()
    assert rel_err(S_scan, S.double().cpu().numpy()) <= tol
