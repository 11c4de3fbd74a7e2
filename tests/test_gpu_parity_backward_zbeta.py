"""GPU parity of the backward pass that takes the value gate as its pre-activation (rodimus_chunk_scan_bwd_zbeta) against
the fp64 backward oracle given the same z_beta bits (needs an MI355X).

Tolerance: max|err| / max|ref| <= 2e-2 per gradient tensor, as for rodimus_chunk_scan_bwd (dz_beta is rounded to bf16)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, rel_err, to_dev

pytestmark = pytest.mark.gpu


def _case(B, T, H, dv, s0=True, seed=0, **kw):
    w = wl.ScanWorkload("case", B=B, T=T, H=H, dk=64, dv=dv, chunk=64, io_dtype="bf16", s0_std=0.1 if s0 else 0.0, seed=seed, **kw)
    inp = wl.make_scan_inputs(w)
    rng = np.random.Generator(np.random.PCG64(seed + 2000))
    inp["d_o"] = torch.from_numpy(rng.standard_normal((B, T, H, dv), dtype=np.float32)).to(torch.bfloat16)
    inp["dS_T"] = torch.from_numpy(rng.standard_normal((B, H, 64, dv), dtype=np.float32) * np.float32(0.1))
    return inp


def _check(inp, label, with_dS=True):
    g = to_dev(inp)
    out = rodimus.rodimus_chunk_scan_bwd_zbeta(g["q"], g["k"], g["v"], g["log_alpha"], g["z_beta"], g["S0"], g["d_o"],
                                               g["dS_T"] if with_dS else None)
    torch.cuda.synchronize()
    ref = oracle.scan_bwd(inp["q"], inp["k"], inp["v"], inp["log_alpha"], None, inp["S0"], inp["d_o"],
                          inp["dS_T"] if with_dS else None, z_beta=inp["z_beta"])
    errs = {name: rel_err(out[name], ref[name]) for name in ("dq", "dk", "dv", "dlog_alpha", "dz_beta", "dS0")}
    print("   " + label + ": " + "  ".join(f"{k} {v:.2e}" for k, v in errs.items()), flush=True)
    for name, e in errs.items():
        assert e <= TOL_BF16, (label, name, e)
    return out, ref


@pytest.mark.parametrize("B,T,H,dv,s0", [
    (1, 16, 1, 128, False),      # one tile
    (2, 200, 2, 256, True),      # ragged tail
    (1, 37, 3, 128, True),
    (1, 1, 1, 256, True),        # single token
    (1, 1000, 2, 256, True),     # cut into four segments: the summary pass evaluates the gate as well
    (2, 520, 1, 128, False),     # three segments, dv = 128
])
def test_shapes(B, T, H, dv, s0):
    print(f"bwd zbeta B{B} T{T} H{H} dv{dv} s0={s0}", flush=True)
    _check(_case(B, T, H, dv, s0, seed=T + dv + 7), f"B{B}T{T}H{H}dv{dv}")


def test_saturated_gates_and_missing_state_cotangent():
    """z_beta = +-60 (gate 1 / gate 0: no gradient reaches the pre-activation) and +-inf, ordinary values elsewhere."""
    inp = _case(1, 100, 2, 128, seed=41)
    z = inp["z_beta"].float()
    z[:, 10:20] = 60.0
    z[:, 30:40] = -60.0
    z[:, 50] = float("inf")
    z[:, 51] = float("-inf")
    inp["z_beta"] = z.to(torch.bfloat16)
    print("bwd zbeta saturated", flush=True)
    out, _ = _check(inp, "saturated", with_dS=False)
    dz = out["dz_beta"].float()
    assert float(dz[:, 10:20].abs().max()) == 0.0          # sigmoid(60) rounds to 1: 1 - gate = 0
    assert float(dz[:, 30:40].abs().max()) < 1e-20         # sigmoid(-60) = 9e-27
    assert float(dz[:, 50:52].abs().max()) == 0.0 and torch.isfinite(dz).all()


def test_agrees_with_the_plain_backward_at_the_same_gate():
    """dq, dk, dv, dlog_alpha, dS0 equal those of rodimus_chunk_scan_bwd at beta = sigmoid(z_beta) up to the rounding of the
    gate, and dz_beta = dbeta .* beta (1 - beta)."""
    inp = _case(2, 130, 2, 256, seed=43)
    g = to_dev(inp)
    a = rodimus.rodimus_chunk_scan_bwd_zbeta(g["q"], g["k"], g["v"], g["log_alpha"], g["z_beta"], g["S0"], g["d_o"], g["dS_T"])
    beta = torch.sigmoid(g["z_beta"].float())
    b = rodimus.rodimus_chunk_scan_bwd(g["q"], g["k"], g["v"], g["log_alpha"], beta, g["S0"], g["d_o"], g["dS_T"])
    for name in ("dq", "dk", "dv", "dlog_alpha", "dS0"):
        assert rel_err(a[name], b[name].float().cpu().numpy().astype(np.float64)) <= 5e-3, name
    chain = (b["dbeta"] * beta * (1 - beta)).cpu().numpy().astype(np.float64)
    assert rel_err(a["dz_beta"], chain) <= 1e-2


def test_refused_outside_the_matrix_core_shapes():
    x = torch.zeros(1, 4, 1, 16, device="cuda:0")
    v = torch.zeros(1, 4, 1, 32, device="cuda:0")
    with pytest.raises(rodimus.RodimusError) as e:
        rodimus.rodimus_chunk_scan_bwd_zbeta(x, x, v, x, v, None, v)
    assert e.value.status == 2
