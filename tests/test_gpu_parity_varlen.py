"""GPU parity of the packed variable-length scan (rodimus_chunk_scan_varlen_fwd) against the fp64 CPU oracle run on
every sequence separately (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, TOL_F32, rel_err, to_dev, tol_for

pytestmark = pytest.mark.gpu


def _oracle_packed(inp, lengths, gate):
    """The definition: the sequential recurrence on each sequence's rows, from that sequence's own initial state."""
    total, H, dv = inp["v"].shape
    dk = inp["q"].shape[-1]
    o = np.zeros((total, H, dv))
    S = np.zeros((len(lengths), H, dk, dv))
    cu = np.concatenate([[0], np.cumsum(lengths)])
    for b, n in enumerate(lengths):
        a, e = int(cu[b]), int(cu[b + 1])
        s0 = None if inp["S0"] is None else inp["S0"][b:b + 1]
        if n == 0:
            S[b] = 0.0 if s0 is None else s0[0].double().numpy()
            continue
        sl = lambda x: x[a:e][None]
        kw = {"z_beta": sl(inp["z_beta"])} if gate == "z_beta" else {}
        beta = sl(inp["beta"]) if gate == "beta" else None
        ob, Sb = oracle.scan(sl(inp["q"]), sl(inp["k"]), sl(inp["v"]), sl(inp["log_alpha"]), beta, s0, **kw)
        o[a:e] = ob[0]
        S[b] = Sb[0]
    return o, S


def _run(inp, gate, chunk, **kw):
    g = to_dev(inp)
    args = {"beta": g["beta"]} if gate == "beta" else ({"z_beta": g["z_beta"]} if gate == "z_beta" else {})
    o, S_T = rodimus.rodimus_chunk_scan_varlen_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], S0=g["S0"],
                                                   chunk=chunk, **args, **kw)
    torch.cuda.synchronize()
    return o, S_T


def _check(lengths, H, dk, dv, chunk, io, gate="beta", s0=True, seed=1):
    inp = wl.make_varlen_inputs(lengths, H, dk, dv, io, s0_std=0.1 if s0 else 0.0, seed=seed)
    o, S_T = _run(inp, gate, chunk)
    o_ref, S_ref = _oracle_packed(inp, lengths, gate)
    tol = tol_for(inp["q"].dtype)
    eo, es = rel_err(o, o_ref), rel_err(S_T, S_ref)
    print(f"   o {eo:.2e}  S_T {es:.2e}", flush=True)
    assert eo <= tol and es <= tol, (eo, es)
    # every sequence on its own as well: a short sequence must not hide behind the global maximum
    go = o.float().cpu().numpy().astype(np.float64)
    cu = np.concatenate([[0], np.cumsum(lengths)])
    for b, n in enumerate(lengths):
        if n:
            ref = o_ref[cu[b]:cu[b + 1]]
            assert np.abs(go[cu[b]:cu[b + 1]] - ref).max() <= tol * max(np.abs(ref).max(), 1e-30), b


@pytest.mark.parametrize("lengths,H,dv,gate,s0", [
    ([64, 128, 192], 2, 128, "beta", True),              # whole chunks
    ([1, 37, 200, 5, 64, 333], 2, 256, "beta", True),    # ragged, shorter than a tile, shorter than a chunk
    ([100, 0, 17, 0], 1, 128, "beta", True),             # empty sequences keep their state
    ([700, 3, 129], 3, 384, "z_beta", False),            # value gate as pre-activation, zero initial states
    ([50, 60], 2, 128, "none", True),                    # no value gate
    ([40, 40, 0, 130, 40, 0, 130, 7], 2, 256, "beta", True),   # equal lengths and empty sequences: the rank by length has ties
    ([3 + (7 * i) % 50 for i in range(70)], 1, 128, "beta", True),   # more than 64 sequences: taken in batch order
    ([1 + (5 * i) % 90 for i in range(64)], 1, 128, "z_beta", True),  # exactly 64: the largest batch that is ranked
])
def test_mfma_path(lengths, H, dv, gate, s0):
    print(f"varlen mfma {lengths} H{H} dv{dv} {gate}", flush=True)
    assert rodimus.rodimus_chunk_scan_path(len(lengths), sum(lengths), H, 64, dv, 64, torch.bfloat16) == rodimus.PATH_MFMA
    _check(lengths, H, 64, dv, 64, "bf16", gate, s0, seed=sum(lengths))


@pytest.mark.parametrize("lengths,H,dk,dv,chunk,io,gate", [
    ([5, 40, 1, 0, 23], 2, 16, 36, 16, "f32", "beta"),
    ([33, 70], 1, 32, 100, 32, "bf16", "z_beta"),
    ([9, 9, 9], 2, 8, 8, 1, "f32", "beta"),
])
def test_generic_path(lengths, H, dk, dv, chunk, io, gate):
    print(f"varlen generic {lengths} H{H} dk{dk} dv{dv} C{chunk} {io} {gate}", flush=True)
    _check(lengths, H, dk, dv, chunk, io, gate, seed=sum(lengths) + dk)


def test_equals_dense_call_when_all_lengths_are_equal():
    B, T, H, dv = 3, 150, 2, 128
    inp = wl.make_varlen_inputs([T] * B, H, 64, dv, "bf16", seed=8)
    print("varlen == dense", flush=True)
    o_p, S_p = _run(inp, "beta", 64)
    g = to_dev(inp)
    r = lambda x: x.reshape(B, T, H, -1)
    o_d, S_d = rodimus.rodimus_chunk_scan_fwd(r(g["q"]), r(g["k"]), r(g["v"]), r(g["log_alpha"]), r(g["beta"]), g["S0"])
    torch.cuda.synchronize()
    assert torch.equal(o_p.reshape(B, T, H, dv), o_d) and torch.equal(S_p, S_d)


def test_state_cache_updated_in_place_then_decode():
    """Prefill a packed batch writing the final states over the initial ones, then continue every sequence with one
    decode step: equals the oracle's scan of each sequence extended by that token."""
    lengths, H, dv = [70, 5, 130], 2, 128
    inp = wl.make_varlen_inputs(lengths, H, 64, dv, "bf16", seed=3)
    tok = wl.make_varlen_inputs([1] * len(lengths), H, 64, dv, "bf16", s0_std=0.0, seed=4)     # one more token each
    g, t = to_dev(inp), to_dev(tok)
    cache = g["S0"].clone()
    print("varlen prefill in place -> decode", flush=True)
    rodimus.rodimus_chunk_scan_varlen_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], beta=g["beta"], S0=cache,
                                          S_T=cache)
    o1 = rodimus.rodimus_decode_step(t["q"], t["k"], t["v"], t["log_alpha"], t["beta"], cache)
    torch.cuda.synchronize()
    _, S_ref = _oracle_packed(inp, lengths, "beta")
    o_ref, S_ref = oracle.step(tok["q"], tok["k"], tok["v"], tok["log_alpha"], tok["beta"], S_ref)
    assert rel_err(o1, o_ref) <= TOL_BF16 and rel_err(cache, S_ref) <= TOL_BF16


def test_corrupt_length_table_stays_inside_the_tensors():
    """Entries outside [0, total] or decreasing are clamped by the kernels: the call completes, outputs are finite for
    the rows a clamped sequence covers, and memory after the tensors is untouched (guard rows keep their fill)."""
    lengths, H, dv = [40, 40, 40], 1, 128
    inp = wl.make_varlen_inputs(lengths, H, 64, dv, "bf16", seed=6)
    g = to_dev(inp)
    total = sum(lengths)
    o = torch.full((total + 64, H, dv), 7.0, dtype=torch.bfloat16, device="cuda:0")
    bad = torch.tensor([-5, 90, 60, 10_000], dtype=torch.int32, device="cuda:0")
    print("varlen corrupt table", flush=True)
    rodimus.rodimus_chunk_scan_varlen_fwd(g["q"], g["k"], g["v"], g["log_alpha"], bad, beta=g["beta"], S0=g["S0"], o=o[:total])
    torch.cuda.synchronize()
    assert torch.all(o[total:] == 7.0)
    assert torch.isfinite(o[:total].float()).all()


def test_serving_mix_full_size():
    """A prefill batch of 48 sequences with a log-uniform length mix, 16384 tokens in total, at the layer's head shape."""
    lengths = wl.serving_length_mix(48, 16384)
    print(f"varlen serving mix: min {min(lengths)} max {max(lengths)}", flush=True)
    _check(lengths, 16, 64, 256, 64, "bf16", "beta", seed=13)


@pytest.mark.parametrize("lengths,H,dk,dv,io", [
    ([37, 1, 0, 130, 16, 65], 2, 64, 128, "bf16"),     # matrix-core kernels: ragged, single-token and empty sequences
    ([200, 33], 2, 64, 256, "bf16"),
    ([9, 0, 20, 1], 2, 16, 32, "f32"),                 # token-by-token kernels
])
def test_packed_backward_matches_the_oracle_per_sequence(lengths, H, dk, dv, io):
    """rodimus_chunk_scan_varlen_bwd against the backward oracle run on every sequence separately."""
    print(f"varlen bwd {lengths} H{H} dk{dk} dv{dv} {io}", flush=True)
    d = wl.make_varlen_inputs(lengths, H, dk, dv, io, seed=sum(lengths) + dv)
    total, N = sum(lengths), len(lengths)
    rng = np.random.Generator(np.random.PCG64(77))
    d_o = torch.from_numpy(rng.standard_normal((total, H, dv), dtype=np.float32))
    d_o = d_o.to(torch.bfloat16) if io == "bf16" else d_o
    dS_T = torch.from_numpy(rng.standard_normal((N, H, dk, dv), dtype=np.float32) * np.float32(0.1))
    g = to_dev(d)
    out = rodimus.rodimus_chunk_scan_varlen_bwd(g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], g["beta"], g["S0"],
                                                d_o.cuda(), dS_T.cuda())
    torch.cuda.synchronize()
    tol_io = TOL_BF16 if io == "bf16" else TOL_F32
    tol_f = TOL_BF16 if io == "bf16" else TOL_F32       # the matrix-core path uses bf16 operands for the fp32 outputs as well
    start = 0
    for b, n in enumerate(lengths):
        sl = slice(start, start + n)
        ref = oracle.scan_bwd(d["q"][sl][None], d["k"][sl][None], d["v"][sl][None], d["log_alpha"][sl][None],
                              d["beta"][sl][None], d["S0"][b][None], d_o[sl][None], dS_T[b][None])
        for name, tol in (("dq", tol_io), ("dk", tol_io), ("dv", tol_io), ("dlog_alpha", tol_f), ("dbeta", tol_f)):
            if n > 0:
                assert rel_err(out[name][sl][None], ref[name]) <= tol, (b, n, name)
        assert rel_err(out["dS0"][b][None], ref["dS0"]) <= tol_f, (b, n, "dS0")
        start += n
