"""GPU parity of the whole-block calls (rodimus_chunk_scan_fwd_gated_block, rodimus_decode_step_gated_block): gates and
pre-processing of Sec. 3.1.2 / 3.1.3, the recurrence, and the output stage of Sec. 3.1.3 in one kernel, against the fp64 oracle
(``scan_gated`` then ``block_output``, both pinned on their own; nothing new is computed on the oracle side).  Needs an MI355X."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, rel_err, to_dev, tol_for

pytestmark = pytest.mark.gpu


def _stage(shape, H, dv, io, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    cast = (lambda a: torch.from_numpy(a).to(torch.bfloat16)) if io == "bf16" else torch.from_numpy
    return {"x_prime": cast(rng.standard_normal(shape, dtype=np.float32)),
            "z_gate": cast(rng.standard_normal(shape, dtype=np.float32) * np.float32(1.5)),
            "d": torch.from_numpy(rng.standard_normal((H, dv), dtype=np.float32))}


@pytest.mark.parametrize("B,T,H,dk,dv,chunk,io,act", [
    (2, 200, 2, 64, 256, 64, "bf16", "silu"),         # matrix-core path, ragged tail, two column tiles
    (1, 1100, 1, 64, 128, 64, "bf16", "sigmoid"),     # matrix-core path, call cut along the sequence
    (2, 70, 3, 16, 36, 16, "f32", "silu"),            # any-shape path
])
def test_scan(B, T, H, dk, dv, chunk, io, act):
    print(f"gated block scan B{B} T{T} H{H} dk{dk} dv{dv} {io} {act}", flush=True)
    d = wl.make_gated_scan_inputs(B, T, H, dk, dv, io, seed=T)
    st = _stage((B, T, H, dv), H, dv, io, T + 1)
    g, gs = to_dev(d), to_dev(st)
    y, S_T = rodimus.rodimus_chunk_scan_fwd_gated_block(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["z_beta"], g["S0"], chunk=chunk,
                                                        x_prime=gs["x_prime"], d=gs["d"], z_gate=gs["z_gate"], gate_act=act)
    torch.cuda.synchronize()
    o_ref, S_ref = oracle.scan_gated(d["q"], d["k"], d["v"], d["z_g"], d["z_tau"], d["z_beta"], d["S0"])
    y_ref = oracle.block_output(o_ref, st["x_prime"], st["d"], st["z_gate"], act)
    tol = tol_for(d["q"].dtype)
    ey, es = rel_err(y, y_ref), rel_err(S_T, S_ref)
    print(f"   y {ey:.2e}  S_T {es:.2e}", flush=True)
    assert ey <= tol and es <= tol
    # the same call without the stage is the gated scan itself, bit for bit
    o_plain, _ = rodimus.rodimus_chunk_scan_fwd_gated(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["z_beta"], g["S0"], chunk=chunk)
    o_nostage, _ = rodimus.rodimus_chunk_scan_fwd_gated_block(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["z_beta"], g["S0"], chunk=chunk)
    assert torch.equal(o_plain.view(torch.int16 if io == "bf16" else torch.int32), o_nostage.view(torch.int16 if io == "bf16" else torch.int32))


@pytest.mark.parametrize("N,H,dk,dv,io", [(5, 3, 64, 256, "bf16"), (2, 2, 16, 32, "f32")])
def test_decode_steps_chain_from_the_scan(N, H, dk, dv, io):
    print(f"gated block decode N{N} H{H} dk{dk} dv{dv} {io}", flush=True)
    T = 5
    d = wl.make_gated_scan_inputs(N, T, H, dk, dv, io, seed=31)
    st = _stage((N, T, H, dv), H, dv, io, 32)
    g, gs = to_dev(d), to_dev(st)
    S = g["S0"].clone()
    ys = []
    for t in range(T):
        ys.append(rodimus.rodimus_decode_step_gated_block(g["q"][:, t].contiguous(), g["k"][:, t].contiguous(), g["v"][:, t].contiguous(),
                                                          g["z_g"][:, t].contiguous(), g["z_tau"][:, t].contiguous(),
                                                          g["z_beta"][:, t].contiguous(), S, x_prime=gs["x_prime"][:, t].contiguous(),
                                                          d=gs["d"], z_gate=gs["z_gate"][:, t].contiguous(), gate_act="silu"))
    torch.cuda.synchronize()
    o_ref, S_ref = oracle.scan_gated(d["q"], d["k"], d["v"], d["z_g"], d["z_tau"], d["z_beta"], d["S0"])
    y_ref = oracle.block_output(o_ref, st["x_prime"], st["d"], st["z_gate"], "silu")
    tol = tol_for(d["q"].dtype)
    assert rel_err(torch.stack(ys, 1), y_ref) <= tol and rel_err(S, S_ref) <= tol


def test_full_size_layer_config():
    """The layer-shaped configuration at full size (the launch that bench.py times as scan_whole_block), every output element
    and every final state against the oracle, with a bar per (batch, head) as well."""
    w = wl.LAYER_1P6B
    print("gated block layer_1p6b: inputs ...", flush=True)
    d = wl.make_gated_scan_inputs(w.B, w.T, w.H, w.dk, w.dv, "bf16", seed=17)
    st = _stage((w.B, w.T, w.H, w.dv), w.H, w.dv, "bf16", 21)
    g, gs = to_dev(d), to_dev(st)
    print("gated block layer_1p6b: GPU ...", flush=True)
    y, S_T = rodimus.rodimus_chunk_scan_fwd_gated_block(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["z_beta"], g["S0"], chunk=w.chunk,
                                                        x_prime=gs["x_prime"], d=gs["d"], z_gate=gs["z_gate"], gate_act="silu")
    torch.cuda.synchronize()
    print("gated block layer_1p6b: oracle ...", flush=True)
    o_ref, S_ref = oracle.scan_gated(d["q"], d["k"], d["v"], d["z_g"], d["z_tau"], d["z_beta"], d["S0"])
    y_ref = oracle.block_output(o_ref, st["x_prime"], st["d"], st["z_gate"], "silu")
    del o_ref
    ey, es = rel_err(y, y_ref), rel_err(S_T, S_ref)
    print(f"   y {ey:.2e}  S_T {es:.2e}", flush=True)
    assert ey <= TOL_BF16 and es <= TOL_BF16
    gy = y.float().cpu().numpy()
    for b in range(w.B):
        for h in range(w.H):
            ref = y_ref[b, :, h]
            assert np.abs(gy[b, :, h] - ref).max() <= TOL_BF16 * np.abs(ref).max(), (b, h)
