"""The scan entry point that allocates nothing (rodimus_chunk_scan_fwd_noalloc) against rodimus_chunk_scan_fwd, which takes
the same call's workspace from the caller: two calls in a row through the C ABI, the second on a smaller input, so that the
second finds the first call's contents in the library's built-in scratch buffer."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, rel_err, to_dev

pytestmark = pytest.mark.gpu


def _both(w):
    inp = wl.make_scan_inputs(w)
    g = to_dev(inp)
    need = rodimus.rodimus_chunk_scan_workspace_bytes(w.B, w.T, w.H, w.dk, w.dv, w.chunk, torch.bfloat16)
    o_ref, S_ref = rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], chunk=w.chunk)
    o = torch.full_like(o_ref, float("nan"))
    S_T = torch.full_like(S_ref, float("nan"))
    rodimus.rodimus_chunk_scan_fwd_noalloc(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], o, S_T, chunk=w.chunk)
    torch.cuda.synchronize()
    return inp, need, (o, S_T), (o_ref, S_ref)


def test_two_calls_in_a_row_second_one_smaller():
    first = wl.shrink(wl.LONG_CONTEXT, T=8192)                        # B=1, H=16, dv=256: cut into 8 segments, 8 MB of scratch
    second = wl.shrink(wl.LAYER_1P6B, B=2, T=1024, H=4, dv=128)       # cut into 4 segments, 1 MB of scratch, non-zero S0
    assert rodimus.lib().rodimus_chunk_scan_fwd_noalloc_scratch_bytes() == 10 << 20
    for w in (first, second):
        inp, need, got, ref = _both(w)
        assert 0 < need <= 10 << 20, (w, need)                        # the call does use the scratch buffer
        # same kernels on the same inputs: identical bits
        assert torch.equal(got[0].view(torch.int16), ref[0].view(torch.int16)), w.name
        assert torch.equal(got[1].view(torch.int32), ref[1].view(torch.int32)), w.name
        o_orc, S_orc = oracle.scan(inp["q"], inp["k"], inp["v"], inp["log_alpha"], inp["beta"], inp["S0"])
        assert rel_err(got[0], o_orc) <= TOL_BF16 and rel_err(got[1], S_orc) <= TOL_BF16


def test_call_without_scratch_and_without_state():
    w = wl.shrink(wl.LAYER_1P6B, B=2, T=200, H=2)                     # too short to be cut: no scratch
    inp = wl.make_scan_inputs(w)
    g = to_dev(inp)
    o_ref, _ = rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], chunk=w.chunk)
    o = torch.empty_like(o_ref)
    rodimus.rodimus_chunk_scan_fwd_noalloc(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], o, None, chunk=w.chunk)
    torch.cuda.synchronize()
    assert torch.equal(o.view(torch.int16), o_ref.view(torch.int16))
