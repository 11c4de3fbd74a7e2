"""NaN and Inf in the inputs (needs an MI355X): every kernel returns, and a non-finite value stays inside the (batch, head)
recurrence it was fed to -- the other recurrences of the same call produce the same bits as without it.  (Every (batch, head)
is an independent recurrence in the paper's formulation, Sec. 3.1.3; a kernel that let NaN leak across them through a shared
tile or a reduction would break that.)"""
import pytest
import torch

from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import to_dev

pytestmark = pytest.mark.gpu


def _same_bits(a, b):
    return torch.equal(a.contiguous().view(torch.int16 if a.dtype == torch.bfloat16 else torch.int32),
                       b.contiguous().view(torch.int16 if b.dtype == torch.bfloat16 else torch.int32))


def _others_untouched(clean, dirty, b, h, head_axis):
    """Every (batch, head) but (b, h) has the same bits in both results; returns the dirty result's slice at (b, h)."""
    B, H = clean.shape[0], clean.shape[head_axis]
    for bb in range(B):
        for hh in range(H):
            if (bb, hh) != (b, h):
                assert _same_bits(clean[bb].select(head_axis - 1, hh), dirty[bb].select(head_axis - 1, hh)), (bb, hh)
    return dirty[b].select(head_axis - 1, h)


@pytest.mark.parametrize("T,dv", [(300, 256), (1100, 128)])          # single pass; call cut along the sequence
@pytest.mark.parametrize("where,value", [("v", float("nan")), ("log_alpha", float("nan")), ("q", float("inf")),
                                         ("beta", float("-inf")), ("k", float("nan"))])
def test_forward_scan_contains_non_finite_values(T, dv, where, value):
    w = wl.shrink(wl.LAYER_1P6B, B=2, T=T, H=3, dv=dv)
    inp = wl.make_scan_inputs(w)
    g = to_dev(inp)
    o0, S0 = rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], chunk=64)
    b, h, t = 1, 2, 77
    g[where][b, t, h, 5] = value
    o1, S1 = rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], chunk=64)
    torch.cuda.synchronize()                                     # the kernels came back
    bad_o = _others_untouched(o0, o1, b, h, 2)
    _others_untouched(S0, S1, b, h, 1)
    # nothing travels back beyond the 16-row tile of the recurrence that holds row t (inside the tile the masked scores
    # multiply the bad row by zero, and 0 * NaN is NaN: earlier rows of that tile may be hit)
    assert _same_bits(bad_o[:t - t % 16], o0[b, :t - t % 16, h])
    assert not torch.isfinite(bad_o[t:].float()).all()           # the value did arrive where it belongs


def test_gated_and_block_forms_contain_non_finite_values():
    d = wl.make_gated_scan_inputs(2, 260, 2, 64, 256, "bf16", seed=4)
    g = to_dev(d)
    o0, S0 = rodimus.rodimus_chunk_scan_fwd_gated(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["z_beta"], g["S0"])
    g["z_g"][0, 100, 1, 9] = float("nan")
    g["z_beta"][0, 130, 1, 200] = float("inf")                   # sigmoid(+inf) = 1: finite result, still only there
    o1, S1 = rodimus.rodimus_chunk_scan_fwd_gated(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["z_beta"], g["S0"])
    torch.cuda.synchronize()
    _others_untouched(o0, o1, 0, 1, 2)
    _others_untouched(S0, S1, 0, 1, 1)
    w = wl.shrink(wl.LAYER_1P6B, B=2, T=200, H=2)
    g = to_dev(wl.make_scan_inputs(w))
    x = torch.randn((2, 200, 2, 256), device="cuda:0").to(torch.bfloat16)
    z = torch.randn((2, 200, 2, 256), device="cuda:0").to(torch.bfloat16)
    dd = torch.randn((2, 256), device="cuda:0")
    run = lambda: rodimus.rodimus_chunk_scan_fwd_block(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], x_prime=x, d=dd,
                                                       z_gate=z, gate_act="silu")
    o0, S0 = run()
    x[1, 50, 0, 3] = float("nan")                                # the feed-through touches one output element only
    o1, S1 = run()
    torch.cuda.synchronize()
    assert _same_bits(S0, S1)
    bad = torch.isnan(o1.float()) != torch.isnan(o0.float())
    assert int(bad.sum()) == 1 and bool(bad[1, 50, 0, 3])


def test_decode_step_contains_non_finite_values():
    dw = wl.DecodeWorkload("nonfinite", N=6, H=4, dk=64, dv=256, steps=2, ring=2)
    d = wl.make_decode_inputs(dw)
    tok = to_dev(d["ring"][0])
    Sa, Sb = d["S"].to("cuda:0"), d["S"].to("cuda:0")
    oa = rodimus.rodimus_decode_step(tok["q"], tok["k"], tok["v"], tok["log_alpha"], tok["beta"], Sa)
    tok["k"][3, 2, 7] = float("nan")
    tok["log_alpha"][4, 0, 1] = float("inf")
    ob = rodimus.rodimus_decode_step(tok["q"], tok["k"], tok["v"], tok["log_alpha"], tok["beta"], Sb)
    torch.cuda.synchronize()
    for n in range(6):
        for h in range(4):
            if (n, h) in ((3, 2), (4, 0)):
                assert not torch.isfinite(Sb[n, h]).all()
            else:
                assert _same_bits(Sa[n, h], Sb[n, h]) and _same_bits(oa[n, h], ob[n, h]), (n, h)


def test_backward_contains_non_finite_values():
    w = wl.shrink(wl.LAYER_1P6B, B=2, T=300, H=2, dv=128)
    inp = wl.make_scan_inputs(w)
    g = to_dev(inp)
    d_o = torch.randn((2, 300, 2, 128), device="cuda:0").to(torch.bfloat16)
    run = lambda: rodimus.rodimus_chunk_scan_bwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], d_o)
    clean = run()
    d_o[1, 200, 0, 17] = float("nan")
    g["v"][0, 10, 1, 3] = float("inf")
    dirty = run()
    torch.cuda.synchronize()
    for name, axis in (("dq", 2), ("dk", 2), ("dv", 2), ("dlog_alpha", 2), ("dbeta", 2), ("dS0", 1)):
        for b in range(2):
            for h in range(2):
                if (b, h) in ((1, 0), (0, 1)):
                    continue
                assert _same_bits(clean[name][b].select(axis - 1, h), dirty[name][b].select(axis - 1, h)), (name, b, h)
    assert not torch.isfinite(dirty["dq"][1, :, 0].float()).all()
