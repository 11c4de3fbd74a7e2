"""GPU parity of the bf16 MFMA chunk-scan kernel against the fp64 CPU oracle (needs an MI355X).

Tolerance: max|err| / max|ref| <= 2e-2 for o and for S_T separately (bf16 inputs and outputs, fp32 state)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, check_scan, gpu_scan, oracle_scan, rel_err, to_dev

pytestmark = pytest.mark.gpu


def _case(B, T, H, dv, s0=True, seed=0, **kw):
    w = wl.ScanWorkload("case", B=B, T=T, H=H, dk=64, dv=dv, chunk=64, io_dtype="bf16",
                        s0_std=0.1 if s0 else 0.0, seed=seed, **kw)
    return wl.make_scan_inputs(w)


def test_path_selection():
    assert rodimus.rodimus_chunk_scan_path(8, 4096, 16, 64, 256, 64, torch.bfloat16) == rodimus.PATH_MFMA
    assert rodimus.rodimus_chunk_scan_path(4, 2048, 8, 64, 128, 64, torch.bfloat16) == rodimus.PATH_MFMA
    assert rodimus.rodimus_chunk_scan_path(4, 2048, 8, 64, 128, 32, torch.bfloat16) == rodimus.PATH_GENERIC
    assert rodimus.rodimus_chunk_scan_path(4, 2048, 8, 64, 128, 64, torch.float32) == rodimus.PATH_GENERIC


@pytest.mark.parametrize("B,T,H,dv,s0", [
    (1, 64, 1, 128, False),      # one chunk, one tile
    (1, 128, 2, 128, True),      # two chunks: state carried once
    (2, 200, 3, 256, True),      # several chunks, ragged tail (200 = 3*64 + 8), two column tiles
    (1, 37, 2, 128, True),       # shorter than one chunk
    (1, 1, 1, 128, True),        # single token
    (2, 640, 2, 384, False),     # three column tiles, ten chunks
])
def test_small_shapes(B, T, H, dv, s0):
    print(f"mfma B{B} T{T} H{H} dv{dv} s0={s0}", flush=True)
    inp = _case(B, T, H, dv, s0, seed=T + dv)
    eo, es = check_scan(inp, 64, f"B{B}T{T}H{H}dv{dv}")
    print(f"   o {eo:.2e}  S_T {es:.2e}", flush=True)


@pytest.mark.parametrize("B,T,H,dv", [
    (9, 130, 15, 256),           # 135 (batch, head) pairs x 2 column tiles = 270 workgroups; 135 is not a multiple of 8
    (6, 70, 15, 384),            # 90 pairs x 3 column tiles
])
def test_more_workgroups_than_compute_units(B, T, H, dv):
    """Dense batches with more than 256 workgroups run on a flat grid that keeps the column tiles of a (batch, head) on one
    XCD; the grid is rounded up to whole runs of eight pairs."""
    print(f"mfma flat grid B{B} T{T} H{H} dv{dv}", flush=True)
    assert rodimus.rodimus_chunk_scan_workspace_bytes(B, T, H, 64, dv, 64, torch.bfloat16) == 0      # not the split path
    inp = _case(B, T, H, dv, True, seed=B + dv)
    eo, es = check_scan(inp, 64, f"flat B{B}T{T}H{H}dv{dv}")
    print(f"   o {eo:.2e}  S_T {es:.2e}", flush=True)


@pytest.mark.parametrize("B,T,H,dv,s0", [
    (1, 640, 2, 384, True),      # 10 chunks -> 2 segments of 5
    (1, 581, 1, 128, True),      # ragged last segment
    (2, 1100, 1, 256, False),    # 18 chunks -> 4 segments (5,5,5,3), ragged tail, zero initial state
    (1, 4096, 2, 128, True),     # 64 chunks -> 16 segments
])
def test_sequence_split_path(B, T, H, dv, s0):
    """Few (batch, head, column tile) triples: the call is cut into sequence segments (summary pass, segment scan,
    main pass) and must still match the oracle; the final state may be written over the initial one."""
    need = rodimus.rodimus_chunk_scan_workspace_bytes(B, T, H, 64, dv, 64, torch.bfloat16)
    assert need > 0, "shape chosen to take the split path"
    print(f"split B{B} T{T} H{H} dv{dv}: workspace {need} B", flush=True)
    inp = _case(B, T, H, dv, s0, seed=T)
    eo, es = check_scan(inp, 64, f"split B{B}T{T}H{H}dv{dv}")
    print(f"   o {eo:.2e}  S_T {es:.2e}", flush=True)
    if s0:
        g = to_dev(inp)
        state = g["S0"].clone()
        o, _ = rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], state, chunk=64, S_T=state)
        torch.cuda.synchronize()
        o_ref, S_ref = oracle_scan(inp)
        assert rel_err(o, o_ref) <= TOL_BF16 and rel_err(state, S_ref) <= TOL_BF16


def test_split_path_rejects_small_workspace():
    inp = _case(1, 640, 2, 384, seed=3)
    g = to_dev(inp)
    need = rodimus.rodimus_chunk_scan_workspace_bytes(1, 640, 2, 64, 384, 64, torch.bfloat16)
    small = torch.empty(need - 16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(rodimus.RodimusError) as e:
        rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], chunk=64, workspace=small)
    assert e.value.status == 5


def test_beta_none_alpha_one_is_causal_linear_attention():
    inp = _case(1, 192, 2, 128, s0=False, seed=4)
    inp["beta"] = None
    inp["log_alpha"].zero_()
    check_scan(inp, 64, "alpha=1,beta=1")


def test_hard_resets_and_extreme_decay():
    """alpha = 0 inside tiles, and decays whose quotient form would overflow bf16/fp32, stay finite and in tolerance."""
    inp = _case(1, 256, 2, 128, seed=6)
    la = inp["log_alpha"]
    la[0, 5, 0, :] = -float("inf")
    la[0, 70, 0, 3] = -float("inf")
    la[0, 100:108, 1, 9] = -float("inf")
    la[0, 130:190, 1, 7] = -30.0          # 60 steps of exp(-30) across a chunk boundary
    la[0, 200:232, 0, :] = -12.0          # a whole half chunk of strong decay on every channel
    o, S_T = gpu_scan(inp, 64)
    assert torch.isfinite(o.float()).all() and torch.isfinite(S_T).all()
    o_ref, S_ref = oracle_scan(inp)
    assert rel_err(o, o_ref) <= TOL_BF16 and rel_err(S_T, S_ref) <= TOL_BF16


@pytest.mark.parametrize("la_value", [-3.3, -3.4, -3.5, -3.6, -8.0])
def test_both_tile_constructions_around_the_switch(la_value):
    """A 16-row tile uses the quotient form of the pairwise decay while its total decay stays above 2^-80 and the
    product-only form below.  Constant log_alpha of -3.4 / -3.5 per step puts the tile total just above / below
    that switch (exp(-16*3.4) = 2^-78.5, exp(-16*3.5) = 2^-80.8); both sides must agree with the oracle."""
    inp = _case(1, 192, 2, 128, seed=12)
    inp["log_alpha"][..., ::2] = la_value          # every other channel strongly decayed, the rest as drawn
    eo, es = check_scan(inp, 64, f"la={la_value}")
    print(f"la {la_value}: o {eo:.2e} S_T {es:.2e}", flush=True)


def test_alpha_zero_everywhere():
    inp = _case(1, 128, 1, 128, seed=2)
    inp["log_alpha"].fill_(-float("inf"))
    check_scan(inp, 64, "alpha=0")


def test_split_sequence_resume_and_state_aliasing():
    inp = _case(2, 320, 2, 128, seed=8)
    o_ref, S_ref = oracle_scan(inp)
    g = to_dev(inp)
    T1 = 128
    sl = lambda x, a, b: x[:, a:b].contiguous()
    state = g["S0"].clone()
    o1, _ = rodimus.rodimus_chunk_scan_fwd(sl(g["q"], 0, T1), sl(g["k"], 0, T1), sl(g["v"], 0, T1),
                                           sl(g["log_alpha"], 0, T1), sl(g["beta"], 0, T1), state, chunk=64, S_T=state)
    o2, _ = rodimus.rodimus_chunk_scan_fwd(sl(g["q"], T1, 320), sl(g["k"], T1, 320), sl(g["v"], T1, 320),
                                           sl(g["log_alpha"], T1, 320), sl(g["beta"], T1, 320), state, chunk=64, S_T=state)
    torch.cuda.synchronize()
    assert rel_err(torch.cat([o1, o2], dim=1), o_ref) <= TOL_BF16
    assert rel_err(state, S_ref) <= TOL_BF16


def test_outputs_stay_inside_their_buffers_and_are_deterministic():
    inp = _case(1, 100, 2, 128, seed=13)
    g = to_dev(inp)
    pad = 64
    o_buf = torch.full((100 * 2 * 128 + 2 * pad,), 7.0, device="cuda:0", dtype=torch.bfloat16)
    s_buf = torch.full((2 * 64 * 128 + 2 * pad,), 7.0, device="cuda:0")
    o = o_buf[pad:-pad].view(1, 100, 2, 128)
    S_T = s_buf[pad:-pad].view(1, 2, 64, 128)
    rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], chunk=64, o=o, S_T=S_T)
    o2, S2 = rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], chunk=64)
    torch.cuda.synchronize()
    for buf in (o_buf, s_buf):
        assert (buf[:pad] == 7.0).all() and (buf[-pad:] == 7.0).all()
    assert torch.equal(o, o2) and torch.equal(S_T, S2)
    o_ref, S_ref = oracle_scan(inp)
    assert rel_err(o, o_ref) <= TOL_BF16 and rel_err(S_T, S_ref) <= TOL_BF16


def test_matches_generic_kernel_and_chained_decode():
    """Chunkwise (MFMA) == chunkwise (generic, other chunk size) == recurrent decode, all within tolerance of the oracle."""
    inp = _case(1, 128, 2, 128, seed=21)
    o_ref, S_ref = oracle_scan(inp)
    o_m, S_m = gpu_scan(inp, 64)
    o_g, S_g = gpu_scan(inp, 32)          # chunk 32 runs the generic kernel
    g = to_dev(inp)
    S = g["S0"].clone()
    outs = [rodimus.rodimus_decode_step(*(g[x][:, t].contiguous() for x in ("q", "k", "v", "log_alpha", "beta")), S)
            for t in range(128)]
    torch.cuda.synchronize()
    for o_x, S_x in ((o_m, S_m), (o_g, S_g), (torch.stack(outs, dim=1), S)):
        assert rel_err(o_x, o_ref) <= TOL_BF16 and rel_err(S_x, S_ref) <= TOL_BF16


def test_mid_config_full():
    """Second configuration of the baseline file, full size, every output compared."""
    inp = wl.make_scan_inputs(wl.MID)
    print("mid config: oracle ...", flush=True)
    eo, es = check_scan(inp, wl.MID.chunk, "mid")
    print(f"mid: o {eo:.2e}  S_T {es:.2e}", flush=True)
