"""GPU parity of the whole block over a packed variable-length batch (rodimus_chunk_scan_varlen_fwd_gated_block) against the fp64
oracle run on every sequence separately: ``scan_gated`` on the sequence's rows from its own initial state, then ``block_output``
(both pinned on their own; nothing new is computed on the oracle side).  Needs an MI355X."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import rel_err, to_dev, tol_for

pytestmark = pytest.mark.gpu


def _inputs(lengths, H, dk, dv, io, seed):
    total, N = int(sum(lengths)), len(lengths)
    d = wl.make_gated_scan_inputs(1, max(total, 1), H, dk, dv, io, s0_std=0.0, seed=seed)
    d = {k: (None if v is None else v[0, :total]) for k, v in d.items()}
    rng = np.random.Generator(np.random.PCG64(seed + 7))
    cast = (lambda a: torch.from_numpy(a).to(torch.bfloat16)) if io == "bf16" else torch.from_numpy
    d["x_prime"] = cast(rng.standard_normal((total, H, dv), dtype=np.float32))
    d["z_gate"] = cast(rng.standard_normal((total, H, dv), dtype=np.float32) * np.float32(1.5))
    d["d"] = torch.from_numpy(rng.standard_normal((H, dv), dtype=np.float32))
    d["S0"] = torch.from_numpy(rng.standard_normal((N, H, dk, dv), dtype=np.float32) * np.float32(0.1))
    cu = np.zeros(N + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    d["cu_seqlens"] = torch.from_numpy(cu)
    return d


def _oracle(d, lengths, act, stage=True):
    total, H, dv = d["v"].shape
    y = np.zeros((total, H, dv))
    S = d["S0"].double().numpy().copy()
    cu = d["cu_seqlens"].numpy()
    for b, n in enumerate(lengths):
        if n == 0:
            continue
        a, e = int(cu[b]), int(cu[b + 1])
        sl = lambda x: x[a:e][None]
        o_b, S_b = oracle.scan_gated(sl(d["q"]), sl(d["k"]), sl(d["v"]), sl(d["z_g"]), sl(d["z_tau"]), sl(d["z_beta"]), d["S0"][b:b + 1])
        y[a:e] = oracle.block_output(o_b, sl(d["x_prime"]), d["d"], sl(d["z_gate"]), act)[0] if stage else o_b[0]
        S[b] = S_b[0]
    return y, S


def _check(lengths, H, dk, dv, chunk, io, act, cut, seed):
    d = _inputs(lengths, H, dk, dv, io, seed)
    g = to_dev(d)
    y, S_T = rodimus.rodimus_chunk_scan_varlen_fwd_gated_block(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["cu_seqlens"], g["z_beta"],
                                                               g["S0"], x_prime=g["x_prime"], d=g["d"], z_gate=g["z_gate"], gate_act=act,
                                                               chunk=chunk, cut=cut)
    torch.cuda.synchronize()
    y_ref, S_ref = _oracle(d, lengths, act)
    tol = tol_for(d["q"].dtype)
    ey, es = rel_err(y, y_ref), rel_err(S_T, S_ref)
    print(f"   y {ey:.2e}  S_T {es:.2e}", flush=True)
    assert ey <= tol and es <= tol
    gy = y.float().cpu().numpy().astype(np.float64)
    cu = d["cu_seqlens"].numpy()
    for b, n in enumerate(lengths):          # every sequence on its own: a short one must not hide behind the global maximum
        if n:
            ref = y_ref[cu[b]:cu[b + 1]]
            assert np.abs(gy[cu[b]:cu[b + 1]] - ref).max() <= tol * max(np.abs(ref).max(), 1e-30), b


@pytest.mark.parametrize("lengths,H,dv,act,cut", [
    ([1, 37, 200, 0, 64, 333], 2, 256, "silu", False),       # ragged, empty, shorter than a tile; one workgroup set per sequence
    ([700, 3, 129], 3, 128, "sigmoid", False),
    ([2900, 0, 1500, 77], 2, 256, "silu", True),             # cut into segments of 512 tokens by the kernels
    ([1024, 512, 513], 1, 128, "sigmoid", True),
])
def test_mfma_path(lengths, H, dv, act, cut):
    print(f"varlen gated block {lengths} H{H} dv{dv} {act} cut={cut}", flush=True)
    if cut:
        assert rodimus.rodimus_chunk_scan_varlen_workspace_bytes(len(lengths), sum(lengths), H, 64, dv, 64, torch.bfloat16) > 0
    _check(lengths, H, 64, dv, 64, "bf16", act, cut, seed=sum(lengths))


def test_generic_path():
    print("varlen gated block generic", flush=True)
    _check([5, 40, 1, 0, 23], 2, 16, 36, 16, "f32", "silu", False, seed=9)


def test_without_stage_inputs_is_the_packed_gated_scan_and_updates_the_cache_in_place():
    lengths, H, dv = [150, 20, 0, 90], 2, 128
    d = _inputs(lengths, H, 64, dv, "bf16", seed=5)
    g = to_dev(d)
    cache = g["S0"].clone()
    print("varlen gated, no stage, in place", flush=True)
    o, S_T = rodimus.rodimus_chunk_scan_varlen_fwd_gated_block(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["cu_seqlens"], g["z_beta"],
                                                               cache, S_T=cache)
    torch.cuda.synchronize()
    assert S_T.data_ptr() == cache.data_ptr()
    o_ref, S_ref = _oracle(d, lengths, "sigmoid", stage=False)
    tol = tol_for(d["q"].dtype)
    assert rel_err(o, o_ref) <= tol and rel_err(cache, S_ref) <= tol
