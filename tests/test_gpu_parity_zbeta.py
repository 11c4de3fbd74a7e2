"""GPU parity of the calls that take the value gate as its pre-activation (rodimus_chunk_scan_fwd_zbeta,
rodimus_decode_step_zbeta) against the fp64 CPU oracle given the same z_beta bits (needs an MI355X).

Tolerances as for the calls they mirror: max|err| / max|ref| <= 2e-2 (bf16 I/O), 1e-4 (fp32 I/O)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, TOL_F32, rel_err, to_dev, tol_for

pytestmark = pytest.mark.gpu


def _scan_case(B, T, H, dk, dv, chunk, io, s0=True, seed=0):
    w = wl.ScanWorkload("case", B=B, T=T, H=H, dk=dk, dv=dv, chunk=chunk, io_dtype=io,
                        s0_std=0.1 if s0 else 0.0, seed=seed)
    return wl.make_scan_inputs(w)


def _check(inp, chunk, label):
    g = to_dev(inp)
    o, S_T = rodimus.rodimus_chunk_scan_fwd_zbeta(g["q"], g["k"], g["v"], g["log_alpha"], g["z_beta"], g["S0"], chunk=chunk)
    torch.cuda.synchronize()
    o_ref, S_ref = oracle.scan(inp["q"], inp["k"], inp["v"], inp["log_alpha"], None, inp["S0"], z_beta=inp["z_beta"])
    tol = tol_for(inp["q"].dtype)
    eo, es = rel_err(o, o_ref), rel_err(S_T, S_ref)
    print(f"   {label}: o {eo:.2e}  S_T {es:.2e}", flush=True)
    assert eo <= tol and es <= tol, (label, eo, es)
    return o, S_T


@pytest.mark.parametrize("B,T,H,dv,s0", [
    (1, 64, 1, 128, False),      # one chunk
    (2, 200, 3, 256, True),      # several chunks, ragged tail, two column tiles
    (1, 37, 2, 128, True),       # shorter than one chunk
    (2, 640, 2, 384, False),     # three column tiles, ten chunks
    (1, 1100, 1, 256, True),     # sequence-split path (summary pass, segment scan, main pass), ragged last segment
])
def test_mfma_path(B, T, H, dv, s0):
    print(f"zbeta mfma B{B} T{T} H{H} dv{dv} s0={s0}", flush=True)
    assert rodimus.rodimus_chunk_scan_path(B, T, H, 64, dv, 64, torch.bfloat16) == rodimus.PATH_MFMA
    _check(_scan_case(B, T, H, 64, dv, 64, "bf16", s0, seed=T + dv), 64, "mfma")


def test_mfma_saturated_and_closed_gates():
    """z_beta = +inf / large (gate 1), -inf / very negative (gate 0: the token writes nothing), and ordinary values
    side by side, in every tile of a chunk."""
    inp = _scan_case(1, 256, 2, 64, 128, 64, "bf16", seed=11)
    z = inp["z_beta"].float()
    z[:, 3::7] = float("inf")
    z[:, 5::11] = float("-inf")
    z[:, 6::13] = 40.0
    z[:, 2::17] = -100.0
    inp["z_beta"] = z.to(torch.bfloat16)
    print("zbeta mfma saturated gates", flush=True)
    _check(inp, 64, "saturated")


@pytest.mark.parametrize("B,T,H,dk,dv,chunk,io", [
    (2, 100, 3, 16, 36, 16, "f32"),
    (1, 64, 1, 16, 32, 16, "f32"),
    (2, 96, 2, 32, 100, 32, "bf16"),
])
def test_generic_path(B, T, H, dk, dv, chunk, io):
    print(f"zbeta generic B{B} T{T} H{H} dk{dk} dv{dv} C{chunk} {io}", flush=True)
    _check(_scan_case(B, T, H, dk, dv, chunk, io, seed=T), chunk, "generic")


def test_agrees_with_the_two_call_form():
    """ddts_gates(z_beta) -> beta, then the plain scan: the same result as the fused call up to the rounding of beta."""
    inp = _scan_case(2, 300, 2, 64, 256, 64, "bf16", seed=5)
    g = to_dev(inp)
    print("zbeta vs gates + scan", flush=True)
    o_f, S_f = rodimus.rodimus_chunk_scan_fwd_zbeta(g["q"], g["k"], g["v"], g["log_alpha"], g["z_beta"], g["S0"])
    zero = torch.zeros_like(g["q"])
    _, beta, _, _ = rodimus.rodimus_ddts_gates(zero, zero, g["z_beta"], g["q"], g["k"])
    o_2, S_2 = rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], beta, g["S0"])
    torch.cuda.synchronize()
    assert rel_err(o_f, o_2.float().cpu().numpy()) <= 1e-2          # both outputs are rounded to bf16
    assert rel_err(S_f, S_2.cpu().numpy()) <= 1e-5


@pytest.mark.parametrize("io", ["bf16", "f32"])
def test_decode_step(io):
    w = wl.DecodeWorkload("case", N=5, H=3, dk=64, dv=256, steps=12, ring=4, io_dtype=io, seed=9)
    d = wl.make_decode_inputs(w)
    S = d["S"].to("cuda:0")
    S_ref = d["S"].double().numpy()
    print(f"zbeta decode {io}", flush=True)
    for i in range(w.steps):
        tok = d["ring"][i % w.ring]
        t = to_dev(tok)
        o = rodimus.rodimus_decode_step_zbeta(t["q"], t["k"], t["v"], t["log_alpha"], t["z_beta"], S)
        torch.cuda.synchronize()
        o_ref, S_ref = oracle.step(tok["q"], tok["k"], tok["v"], tok["log_alpha"], None, S_ref, z_beta=tok["z_beta"])
        assert rel_err(o, o_ref) <= tol_for(t["q"].dtype), i
    assert rel_err(S, S_ref) <= TOL_F32


def test_prefill_then_decode_chain():
    """Scan the first part with the fused call, continue token by token with the fused decode step: equals the
    oracle's scan of the whole sequence."""
    inp = _scan_case(2, 150, 2, 64, 128, 64, "bf16", seed=21)
    g = to_dev(inp)
    T0 = 140
    print("zbeta prefill -> decode", flush=True)
    cut = lambda x, a, b: x[:, a:b].contiguous()
    o0, S = rodimus.rodimus_chunk_scan_fwd_zbeta(cut(g["q"], 0, T0), cut(g["k"], 0, T0), cut(g["v"], 0, T0),
                                                 cut(g["log_alpha"], 0, T0), cut(g["z_beta"], 0, T0), g["S0"])
    outs = [o0]
    for t in range(T0, 150):
        o = rodimus.rodimus_decode_step_zbeta(g["q"][:, t].contiguous(), g["k"][:, t].contiguous(), g["v"][:, t].contiguous(),
                                              g["log_alpha"][:, t].contiguous(), g["z_beta"][:, t].contiguous(), S)
        outs.append(o[:, None])
    torch.cuda.synchronize()
    o = torch.cat(outs, dim=1)
    o_ref, S_ref = oracle.scan(inp["q"], inp["k"], inp["v"], inp["log_alpha"], None, inp["S0"], z_beta=inp["z_beta"])
    assert rel_err(o, o_ref) <= TOL_BF16 and rel_err(S, S_ref) <= TOL_BF16


def test_full_size_layer_config():
    """The layer-shaped configuration at full size, every output element against the oracle."""
    w = wl.LAYER_1P6B
    print("zbeta layer_1p6b: inputs ...", flush=True)
    inp = wl.make_scan_inputs(w)
    print("zbeta layer_1p6b: GPU + oracle ...", flush=True)
    _check(inp, w.chunk, "layer_1p6b")
