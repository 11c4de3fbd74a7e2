"""GPU parity of the block's ShortConv (rodimus_short_conv_fwd, rodimus_short_conv_step) against the fp64 oracle
(needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import rel_err, to_dev, TOL_BF16, TOL_F32

pytestmark = pytest.mark.gpu


def _check(B, T, C, W, io, act, use_bias=True, use_state=True, seed=0):
    d = wl.make_short_conv_inputs(B, T, C, W, io, seed)
    g = to_dev(d)
    y, st = rodimus.rodimus_short_conv_fwd(g["x"], g["w"], g["bias"] if use_bias else None,
                                           g["state"] if use_state else None, act=act)
    torch.cuda.synchronize()
    y_ref, st_ref = oracle.short_conv(d["x"], d["w"], d["bias"] if use_bias else None, d["state"] if use_state else None, act)
    tol = TOL_BF16 if io == "bf16" else TOL_F32
    assert rel_err(y, y_ref) <= tol
    # element by element: fp32 arithmetic of W + 1 terms, then one rounding to the output type
    got = y.double().cpu().numpy()
    unit = 2.0 ** -8 if io == "bf16" else 2.0 ** -19
    assert np.all(np.abs(got - y_ref) <= unit * np.maximum(np.abs(y_ref), 1.0))
    # the carried state is a copy of inputs: exact
    assert np.array_equal(st.double().cpu().numpy(), st_ref)
    return y, st


@pytest.mark.parametrize("B,T,C,W,io,act", [
    (2, 100, 256, 4, "bf16", "silu"),       # several runs and a ragged last one
    (1, 33, 4096, 4, "bf16", "silu"),       # the layer's width, two channel blocks, a one-token run
    (3, 64, 40, 3, "f32", "none"),          # fewer channel pieces than a wavefront
    (2, 7, 8, 8, "f32", "silu"),            # widest filter, T shorter than the history
    (2, 65, 64, 2, "bf16", "none"),
    (2, 50, 32, 1, "f32", "silu"),          # no history at all
    (2, 2, 16, 4, "bf16", "silu"),          # T < W - 1: the new state mixes old state and inputs
])
def test_short_conv_matches_the_oracle(B, T, C, W, io, act):
    print(f"short_conv B{B} T{T} C{C} W{W} {io} {act}", flush=True)
    _check(B, T, C, W, io, act, seed=T + C)
    _check(B, T, C, W, io, act, use_bias=False, use_state=False, seed=T + C + 1)


def test_empty_sequence_carries_the_state_over():
    d = wl.make_short_conv_inputs(2, 0, 64, 4, "bf16", 3)
    g = to_dev(d)
    y, st = rodimus.rodimus_short_conv_fwd(g["x"], g["w"], g["bias"], g["state"])
    torch.cuda.synchronize()
    assert y.shape == (2, 0, 64) and torch.equal(st, g["state"])
    y, st = rodimus.rodimus_short_conv_fwd(g["x"], g["w"], g["bias"], None)
    torch.cuda.synchronize()
    assert torch.count_nonzero(st) == 0


@pytest.mark.parametrize("io,W", [("bf16", 4), ("f32", 3)])
def test_decode_steps_match_the_sequence_call_and_the_oracle(io, W):
    N, T, C = 3, 12, 128
    d = wl.make_short_conv_inputs(N, T, C, W, io, 21)
    g = to_dev(d)
    state = g["state"].clone()
    ys = []
    for t in range(T):
        ys.append(rodimus.rodimus_short_conv_step(g["x"][:, t].contiguous(), g["w"], g["bias"], state))
    y_steps = torch.stack(ys, dim=1)
    y_seq, st_seq = rodimus.rodimus_short_conv_fwd(g["x"], g["w"], g["bias"], g["state"])
    torch.cuda.synchronize()
    assert torch.equal(y_steps, y_seq) and torch.equal(state, st_seq)     # same arithmetic in the same order
    y_ref, st_ref = oracle.short_conv(d["x"], d["w"], d["bias"], d["state"], "silu")
    assert rel_err(y_steps, y_ref) <= (TOL_BF16 if io == "bf16" else TOL_F32)
    assert np.array_equal(state.double().cpu().numpy(), st_ref)


def test_prefill_then_decode_handoff():
    # the sequence call leaves the state the decode steps continue from
    B, T, C, W = 2, 40, 256, 4
    d = wl.make_short_conv_inputs(B, T, C, W, "bf16", 8)
    g = to_dev(d)
    y_all, _ = rodimus.rodimus_short_conv_fwd(g["x"], g["w"], g["bias"], None)
    y_pre, st = rodimus.rodimus_short_conv_fwd(g["x"][:, :37].contiguous(), g["w"], g["bias"], None)
    tail = [rodimus.rodimus_short_conv_step(g["x"][:, t].contiguous(), g["w"], g["bias"], st) for t in range(37, T)]
    torch.cuda.synchronize()
    assert torch.equal(torch.cat([y_pre, torch.stack(tail, dim=1)], dim=1), y_all)
