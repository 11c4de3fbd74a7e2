"""GPU parity of the backward pass on the shapes the matrix-core kernels do not cover (fp32 I/O, other key / value
widths): the token-by-token fp32 kernels against the fp64 backward oracle (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, TOL_F32, rel_err, to_dev

pytestmark = pytest.mark.gpu


def _case(B, T, H, dk, dv, io, s0=True, seed=0):
    w = wl.ScanWorkload("case", B=B, T=T, H=H, dk=dk, dv=dv, chunk=16, io_dtype=io, s0_std=0.1 if s0 else 0.0, seed=seed)
    inp = wl.make_scan_inputs(w)
    rng = np.random.Generator(np.random.PCG64(seed + 2000))
    d_o = torch.from_numpy(rng.standard_normal((B, T, H, dv), dtype=np.float32))
    inp["d_o"] = d_o.to(torch.bfloat16) if io == "bf16" else d_o
    inp["dS_T"] = torch.from_numpy(rng.standard_normal((B, H, dk, dv), dtype=np.float32) * np.float32(0.1))
    return inp


def _check(inp, io, label, with_dS=True, with_beta=True):
    g = to_dev(inp)
    out = rodimus.rodimus_chunk_scan_bwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"] if with_beta else None, g["S0"],
                                         g["d_o"], g["dS_T"] if with_dS else None)
    torch.cuda.synchronize()
    ref = oracle.scan_bwd(inp["q"], inp["k"], inp["v"], inp["log_alpha"], inp["beta"] if with_beta else None, inp["S0"],
                          inp["d_o"], inp["dS_T"] if with_dS else None)
    # fp32 arithmetic throughout; with bf16 I/O dq, dk, dv are rounded to bf16 on output
    tol_io = TOL_BF16 if io == "bf16" else TOL_F32
    tols = {"dq": tol_io, "dk": tol_io, "dv": tol_io, "dlog_alpha": TOL_F32, "dbeta": TOL_F32, "dS0": TOL_F32}
    errs = {name: rel_err(out[name], ref[name]) for name in tols if ref[name] is not None}
    print("   " + label + ": " + "  ".join(f"{k} {v:.2e}" for k, v in errs.items()), flush=True)
    for name, e in errs.items():
        assert e <= tols[name], (label, name, e)
    return out, ref


@pytest.mark.parametrize("B,T,H,dk,dv,io", [
    (1, 64, 1, 16, 32, "f32"),        # the small all-fp32 configuration
    (2, 50, 2, 8, 8, "f32"),
    (1, 33, 3, 32, 40, "bf16"),       # odd value width, bf16 I/O
    (2, 70, 2, 64, 128, "f32"),       # the matrix-core shape in fp32 I/O
    (1, 20, 1, 128, 200, "f32"),      # widest key, state near the LDS limit
    (1, 1, 2, 5, 3, "f32"),           # a single token, tiny odd sizes
])
def test_generic_backward_matches_the_oracle(B, T, H, dk, dv, io):
    print(f"bwd generic B{B} T{T} H{H} dk{dk} dv{dv} {io}", flush=True)
    _check(_case(B, T, H, dk, dv, io, seed=T + dv), io, "all inputs")


def test_generic_backward_options_and_closed_gates():
    inp = _case(1, 40, 2, 16, 32, "f32", seed=4)
    print("bwd generic no dS_T / no beta", flush=True)
    _check(inp, "f32", "no dS_T", with_dS=False)
    _check(inp, "f32", "no beta", with_beta=False)
    la = inp["log_alpha"]
    la[:, 5::7] = float("-inf")
    la[:, 20:25] = 0.0
    la[:, 30:33, :, :4] = -40.0
    print("bwd generic closed gates", flush=True)
    out, _ = _check(inp, "f32", "closed gates")
    assert float(out["dlog_alpha"][:, 5::7].abs().max()) == 0.0


def test_generic_backward_empty_sequence_passes_the_state_cotangent_through():
    inp = _case(2, 0, 2, 16, 32, "f32", seed=6)
    g = to_dev(inp)
    out = rodimus.rodimus_chunk_scan_bwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], g["d_o"], g["dS_T"])
    torch.cuda.synchronize()
    assert torch.equal(out["dS0"], g["dS_T"])
