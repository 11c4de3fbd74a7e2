"""GPU parity, generic chunkwise kernel and decode step, against the fp64 CPU oracle (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, TOL_F32, check_scan, gpu_scan, oracle_scan, rel_err, to_dev, tol_for

pytestmark = pytest.mark.gpu


def _case(B, T, H, dk, dv, io="f32", s0=True, seed=0, **kw):
    w = wl.ScanWorkload("case", B=B, T=T, H=H, dk=dk, dv=dv, chunk=16, io_dtype=io,
                        s0_std=0.5 if s0 else 0.0, seed=seed, **kw)
    return wl.make_scan_inputs(w)


def test_tiny_config_fp32():
    """First configuration of the baseline file: B=1 H=1 T=64 dk=16 dv=32 chunk=16, all fp32, tolerance 1e-4."""
    inp = wl.make_scan_inputs(wl.TINY)
    print("tiny config", flush=True)
    eo, es = check_scan(inp, wl.TINY.chunk, "tiny")
    print(f"tiny: o {eo:.2e}  S_T {es:.2e}", flush=True)
    assert rodimus.rodimus_chunk_scan_path(1, 64, 1, 16, 32, 16, torch.float32) == rodimus.PATH_GENERIC


@pytest.mark.parametrize("B,T,H,dk,dv,chunk,io,s0", [
    (2, 100, 3, 16, 36, 16, "f32", True),      # ragged tail (100 = 6*16 + 4), dv not a multiple of the column tile
    (1, 64, 2, 5, 4, 7, "f32", False),         # chunk not a power of two, tiny widths
    (1, 37, 1, 64, 130, 64, "f32", True),      # T shorter than one chunk, three column tiles with a ragged one
    (2, 200, 2, 64, 64, 64, "f32", True),      # full-size chunk, several chunks, ragged tail
    (1, 130, 2, 128, 8, 32, "f32", True),      # widest dk
    (1, 50, 1, 16, 32, 1, "f32", True),        # chunk = 1: the recurrent form
    (2, 96, 2, 32, 100, 32, "bf16", True),     # bf16 I/O through the generic kernel
    (1, 1, 1, 8, 8, 16, "f32", True),          # single token
])
def test_generic_shapes(B, T, H, dk, dv, chunk, io, s0):
    print(f"generic B{B} T{T} H{H} dk{dk} dv{dv} C{chunk} {io}", flush=True)
    inp = _case(B, T, H, dk, dv, io, s0, seed=B * 1000 + T)
    check_scan(inp, chunk, f"B{B}T{T}H{H}dk{dk}dv{dv}C{chunk}{io}")


def test_beta_none_and_state_not_wanted():
    inp = _case(1, 40, 2, 16, 32, seed=5)
    inp["beta"] = None
    check_scan(inp, 16, "beta=None")
    g = to_dev(inp)
    o, S_T = rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], None, g["S0"], chunk=16,
                                            want_state=False)
    torch.cuda.synchronize()
    assert S_T is None
    assert rel_err(o, oracle_scan(inp)[0]) <= TOL_F32


@pytest.mark.parametrize("chunk", [1, 2, 16, 64])
def test_result_does_not_depend_on_chunk(chunk):
    inp = _case(1, 128, 2, 16, 32, seed=11)
    o_ref, S_ref = oracle_scan(inp)
    o, S_T = gpu_scan(inp, chunk)
    assert rel_err(o, o_ref) <= TOL_F32 and rel_err(S_T, S_ref) <= TOL_F32


def test_hard_resets_and_extreme_decay_stay_finite_and_exact():
    """alpha = 0 inside a chunk and decays far beyond the fp32 range of a quotient form."""
    inp = _case(1, 96, 1, 16, 32, seed=21)
    la = inp["log_alpha"]
    la[0, 5, 0, :] = -float("inf")
    la[0, 40, 0, 3] = -float("inf")
    la[0, 60:80, 0, 7] = -30.0            # 20 steps of exp(-30): cumulative decay exp(-600)
    o, S_T = gpu_scan(inp, 32)
    assert torch.isfinite(o).all() and torch.isfinite(S_T).all()
    o_ref, S_ref = oracle_scan(inp)
    assert rel_err(o, o_ref) <= TOL_F32 and rel_err(S_T, S_ref) <= TOL_F32


def test_alpha_zero_everywhere_and_alpha_one_everywhere():
    inp = _case(1, 48, 1, 16, 32, seed=3)
    inp["log_alpha"].fill_(-float("inf"))
    check_scan(inp, 16, "alpha=0")
    inp["log_alpha"].zero_()
    inp["beta"] = None
    check_scan(inp, 16, "alpha=1,beta=1")


def test_split_sequence_resume_and_state_aliasing():
    """S_T of one call is S0 of the next (also when both are the same buffer)."""
    inp = _case(2, 96, 2, 16, 32, seed=8)
    o_ref, S_ref = oracle_scan(inp)
    g = to_dev(inp)
    T1 = 40                                  # not a multiple of the chunk
    sl = lambda x, a, b: x[:, a:b].contiguous()
    state = g["S0"].clone()
    o1, _ = rodimus.rodimus_chunk_scan_fwd(sl(g["q"], 0, T1), sl(g["k"], 0, T1), sl(g["v"], 0, T1),
                                           sl(g["log_alpha"], 0, T1), sl(g["beta"], 0, T1), state, chunk=16, S_T=state)
    o2, _ = rodimus.rodimus_chunk_scan_fwd(sl(g["q"], T1, 96), sl(g["k"], T1, 96), sl(g["v"], T1, 96),
                                           sl(g["log_alpha"], T1, 96), sl(g["beta"], T1, 96), state, chunk=16, S_T=state)
    torch.cuda.synchronize()
    assert rel_err(torch.cat([o1, o2], dim=1), o_ref) <= TOL_F32
    assert rel_err(state, S_ref) <= TOL_F32


def test_outputs_stay_inside_their_buffers():
    """Canary words around o and S_T survive a call."""
    inp = _case(1, 50, 2, 16, 36, seed=13)
    g = to_dev(inp)
    pad = 64
    o_buf = torch.full((50 * 2 * 36 + 2 * pad,), 777.0, device="cuda:0")
    s_buf = torch.full((2 * 16 * 36 + 2 * pad,), 777.0, device="cuda:0")
    o = o_buf[pad:-pad].view(1, 50, 2, 36)
    S_T = s_buf[pad:-pad].view(1, 2, 16, 36)
    rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], chunk=16, o=o, S_T=S_T)
    torch.cuda.synchronize()
    for buf in (o_buf, s_buf):
        assert (buf[:pad] == 777.0).all() and (buf[-pad:] == 777.0).all()
    o_ref, S_ref = oracle_scan(inp)
    assert rel_err(o, o_ref) <= TOL_F32 and rel_err(S_T, S_ref) <= TOL_F32


def test_empty_sequence_copies_the_state():
    S0 = torch.randn(1, 2, 16, 32, device="cuda:0")
    e = lambda d: torch.empty(1, 0, 2, d, device="cuda:0")
    o, S_T = rodimus.rodimus_chunk_scan_fwd(e(16), e(16), e(32), e(16), e(32), S0, chunk=16)
    torch.cuda.synchronize()
    assert o.numel() == 0 and torch.equal(S_T, S0)


# ------------------------------------------------------------------------------------------- decode step
def _decode_case(N, H, dk, dv, io, seed, ring=1):
    return wl.make_decode_inputs(wl.DecodeWorkload("d", N=N, H=H, dk=dk, dv=dv, steps=ring, ring=ring,
                                                   io_dtype=io, seed=seed))


@pytest.mark.parametrize("N,H,dk,dv,io", [
    (3, 2, 64, 256, "bf16"),       # the layer shape of the decode configuration
    (2, 3, 64, 256, "f32"),
    (1, 1, 16, 32, "f32"),         # tiny
    (2, 2, 5, 260, "f32"),         # odd dk, two column tiles with a ragged one
    (1, 2, 256, 8, "bf16"),        # widest dk
    (5, 1, 37, 1028, "bf16"),
])
def test_decode_step(N, H, dk, dv, io):
    print(f"decode N{N} H{H} dk{dk} dv{dv} {io}", flush=True)
    d = _decode_case(N, H, dk, dv, io, seed=N + dk)
    tok = d["ring"][0]
    g = to_dev(tok)
    S = d["S"].to("cuda:0")
    o = rodimus.rodimus_decode_step(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], S)
    torch.cuda.synchronize()
    o_ref, S_ref = oracle.step(tok["q"], tok["k"], tok["v"], tok["log_alpha"], tok["beta"], d["S"])
    tol = TOL_BF16 if io == "bf16" else TOL_F32
    assert rel_err(o, o_ref) <= tol
    assert rel_err(S, S_ref) <= (1e-6 if io == "f32" else tol)      # the state itself stays fp32


def test_decode_streaming_variant_beyond_the_last_level_cache():
    """More than 256 MiB of state switches the kernel to non-temporal accesses; results must not change."""
    N, H = 264, 16                              # 264 * 16 * 64 KiB = 264 MiB of state
    d = _decode_case(N, H, 64, 256, "bf16", seed=31)
    tok = d["ring"][0]
    g = to_dev(tok)
    S = d["S"].to("cuda:0")
    o = rodimus.rodimus_decode_step(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], S)
    torch.cuda.synchronize()
    sub = [0, 1, 131, 262, 263]
    o_ref, S_ref = oracle.step(tok["q"][sub], tok["k"][sub], tok["v"][sub], tok["log_alpha"][sub], tok["beta"][sub],
                               d["S"][sub])
    assert rel_err(o[sub], o_ref) <= TOL_BF16
    assert rel_err(S[sub], S_ref) <= 1e-6


def test_decode_beta_none_and_alpha_zero():
    d = _decode_case(2, 2, 16, 32, "f32", seed=2)
    tok = d["ring"][0]
    tok["log_alpha"][0] = -float("inf")
    g = to_dev(tok)
    S = d["S"].to("cuda:0")
    o = rodimus.rodimus_decode_step(g["q"], g["k"], g["v"], g["log_alpha"], None, S)
    torch.cuda.synchronize()
    o_ref, S_ref = oracle.step(tok["q"], tok["k"], tok["v"], tok["log_alpha"], None, d["S"])
    assert torch.isfinite(S).all()
    assert rel_err(o, o_ref) <= TOL_F32 and rel_err(S, S_ref) <= TOL_F32


def test_chained_decode_steps_equal_the_scan():
    """Recurrent form == chunkwise form: T decode steps reproduce the scan of the same tokens (and the oracle)."""
    inp = _case(2, 48, 2, 16, 32, seed=17)
    o_ref, S_ref = oracle_scan(inp)
    g = to_dev(inp)
    S = g["S0"].clone()
    outs = []
    for t in range(48):
        outs.append(rodimus.rodimus_decode_step(g["q"][:, t].contiguous(), g["k"][:, t].contiguous(),
                                                g["v"][:, t].contiguous(), g["log_alpha"][:, t].contiguous(),
                                                g["beta"][:, t].contiguous(), S))
    torch.cuda.synchronize()
    o_dec = torch.stack(outs, dim=1)
    assert rel_err(o_dec, o_ref) <= TOL_F32 and rel_err(S, S_ref) <= TOL_F32
    o_scan, S_scan = gpu_scan(inp, 16)
    assert rel_err(o_dec, o_scan.double().cpu().numpy()) <= TOL_F32
    assert rel_err(S, S_scan.double().cpu().numpy()) <= TOL_F32


def test_decode_is_deterministic():
    d = _decode_case(4, 2, 64, 256, "bf16", seed=9)
    g = to_dev(d["ring"][0])
    S1, S2 = d["S"].to("cuda:0"), d["S"].to("cuda:0")
    o1 = rodimus.rodimus_decode_step(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], S1)
    o2 = rodimus.rodimus_decode_step(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], S2)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(S1, S2)
