"""GPU parity of the calls with the block's output stage fused (rodimus_chunk_scan_fwd_block, rodimus_decode_step_block):
o = (q S + d .* x') .* act(z), against the fp64 oracle (recurrence, then its output stage) (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, TOL_F32, rel_err, to_dev, tol_for

pytestmark = pytest.mark.gpu


def _stage_inputs(shape, H, dv, io, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    cast = (lambda a: torch.from_numpy(a).to(torch.bfloat16)) if io == "bf16" else torch.from_numpy
    return {"x_prime": cast(rng.standard_normal(shape, dtype=np.float32)),
            "z_gate": cast(rng.standard_normal(shape, dtype=np.float32) * np.float32(1.5)),
            "d": torch.from_numpy(rng.standard_normal((H, dv), dtype=np.float32))}


def _check_scan(B, T, H, dk, dv, chunk, io, act, use_x=True, use_z=True, zbeta=False, seed=0):
    w = wl.ScanWorkload("case", B=B, T=T, H=H, dk=dk, dv=dv, chunk=chunk, io_dtype=io, s0_std=0.1, seed=seed)
    inp = wl.make_scan_inputs(w)
    st = _stage_inputs((B, T, H, dv), H, dv, io, seed + 50)
    g, gs = to_dev(inp), to_dev(st)
    kw = {"z_beta": g["z_beta"]} if zbeta else {"beta": g["beta"]}
    o, S_T = rodimus.rodimus_chunk_scan_fwd_block(g["q"], g["k"], g["v"], g["log_alpha"], S0=g["S0"], chunk=chunk,
                                                  x_prime=gs["x_prime"] if use_x else None, d=gs["d"] if use_x else None,
                                                  z_gate=gs["z_gate"] if use_z else None, gate_act=act, **kw)
    torch.cuda.synchronize()
    okw = {"z_beta": inp["z_beta"]} if zbeta else {}
    o_ref, S_ref = oracle.scan(inp["q"], inp["k"], inp["v"], inp["log_alpha"], None if zbeta else inp["beta"], inp["S0"], **okw)
    y_ref = oracle.block_output(o_ref, st["x_prime"] if use_x else None, st["d"] if use_x else None,
                                st["z_gate"] if use_z else None, act)
    tol = tol_for(inp["q"].dtype)
    eo, es = rel_err(o, y_ref), rel_err(S_T, S_ref)
    print(f"   o {eo:.2e}  S_T {es:.2e}", flush=True)
    assert eo <= tol and es <= tol


@pytest.mark.parametrize("B,T,H,dv,act,use_x,use_z,zbeta", [
    (1, 64, 1, 128, "sigmoid", True, True, False),
    (2, 200, 3, 256, "silu", True, True, False),        # ragged tail, two column tiles
    (1, 300, 2, 128, "sigmoid", True, False, False),    # feed-through only
    (1, 130, 2, 256, "silu", False, True, True),        # output gate only, value gate as pre-activation
    (1, 1100, 1, 256, "silu", True, True, False),       # sequence-split path
])
def test_mfma_path(B, T, H, dv, act, use_x, use_z, zbeta):
    print(f"block mfma B{B} T{T} H{H} dv{dv} {act} x={use_x} z={use_z} zbeta={zbeta}", flush=True)
    _check_scan(B, T, H, 64, dv, 64, "bf16", act, use_x, use_z, zbeta, seed=T)


@pytest.mark.parametrize("B,T,H,dk,dv,chunk,io,act", [
    (2, 100, 3, 16, 36, 16, "f32", "silu"),
    (1, 70, 2, 32, 100, 32, "bf16", "sigmoid"),
])
def test_generic_path(B, T, H, dk, dv, chunk, io, act):
    print(f"block generic B{B} T{T} H{H} dk{dk} dv{dv} {io} {act}", flush=True)
    _check_scan(B, T, H, dk, dv, chunk, io, act, seed=T + dk)


def test_without_any_stage_input_equals_the_plain_call():
    w = wl.ScanWorkload("case", B=1, T=150, H=2, dk=64, dv=128, chunk=64, s0_std=0.1, seed=3)
    g = to_dev(wl.make_scan_inputs(w))
    print("block == plain", flush=True)
    o_b, S_b = rodimus.rodimus_chunk_scan_fwd_block(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"])
    o_p, S_p = rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"])
    torch.cuda.synchronize()
    assert torch.equal(o_b, o_p) and torch.equal(S_b, S_p)


@pytest.mark.parametrize("io,act", [("bf16", "silu"), ("f32", "sigmoid")])
def test_decode_step(io, act):
    w = wl.DecodeWorkload("case", N=4, H=3, dk=64, dv=256, steps=6, ring=3, io_dtype=io, seed=8)
    d = wl.make_decode_inputs(w)
    st = _stage_inputs((w.N, w.H, w.dv), w.H, w.dv, io, 77)
    gs = to_dev(st)
    S = d["S"].to("cuda:0")
    S_ref = d["S"].double().numpy()
    print(f"block decode {io} {act}", flush=True)
    for i in range(w.steps):
        tok = d["ring"][i % w.ring]
        t = to_dev(tok)
        o = rodimus.rodimus_decode_step_block(t["q"], t["k"], t["v"], t["log_alpha"], t["beta"], S, x_prime=gs["x_prime"],
                                              d=gs["d"], z_gate=gs["z_gate"], gate_act=act)
        torch.cuda.synchronize()
        o_ref, S_ref = oracle.step(tok["q"], tok["k"], tok["v"], tok["log_alpha"], tok["beta"], S_ref)
        y_ref = oracle.block_output(o_ref, st["x_prime"], st["d"], st["z_gate"], act)
        assert rel_err(o, y_ref) <= tol_for(t["q"].dtype), i
    assert rel_err(S, S_ref) <= TOL_F32
