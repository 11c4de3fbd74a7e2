"""GPU parity of the backward pass (rodimus_chunk_scan_bwd) against the fp64 backward oracle (needs an MI355X).

Tolerance: max|err| / max|ref| <= 2e-2 per gradient tensor (bf16 inputs, bf16 MFMA operands, fp32 accumulation; dq, dk, dv
are rounded to bf16 on output)."""
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
    rng = np.random.Generator(np.random.PCG64(seed + 1000))
    inp["d_o"] = torch.from_numpy(rng.standard_normal((B, T, H, dv), dtype=np.float32)).to(torch.bfloat16)
    inp["dS_T"] = torch.from_numpy(rng.standard_normal((B, H, 64, dv), dtype=np.float32) * np.float32(0.1))
    return inp


def _check(inp, label, with_dS=True, with_beta=True):
    g = to_dev(inp)
    beta = g["beta"] if with_beta else None
    out = rodimus.rodimus_chunk_scan_bwd(g["q"], g["k"], g["v"], g["log_alpha"], beta, g["S0"], g["d_o"], g["dS_T"] if with_dS else None)
    torch.cuda.synchronize()
    ref = oracle.scan_bwd(inp["q"], inp["k"], inp["v"], inp["log_alpha"], inp["beta"] if with_beta else None, inp["S0"],
                          inp["d_o"], inp["dS_T"] if with_dS else None)
    errs = {}
    for name in ("dq", "dk", "dv", "dlog_alpha", "dbeta", "dS0"):
        if ref[name] is None:
            continue
        errs[name] = rel_err(out[name], ref[name])
    print("   " + label + ": " + "  ".join(f"{k} {v:.2e}" for k, v in errs.items()), flush=True)
    for name, e in errs.items():
        assert e <= TOL_BF16, (label, name, e)
    return out, ref


@pytest.mark.parametrize("B,T,H,dv,s0", [
    (1, 16, 1, 128, False),      # one tile
    (1, 64, 2, 256, True),       # four tiles
    (2, 200, 2, 256, True),      # ragged tail (200 = 12 * 16 + 8)
    (1, 37, 3, 128, True),
    (1, 1, 1, 128, True),        # single token
    (2, 330, 2, 128, False),
])
def test_small_shapes(B, T, H, dv, s0):
    print(f"bwd B{B} T{T} H{H} dv{dv} s0={s0}", flush=True)
    _check(_case(B, T, H, dv, s0, seed=T + dv), f"B{B}T{T}H{H}dv{dv}")


def test_without_state_cotangent_and_without_beta():
    inp = _case(1, 100, 2, 128, seed=5)
    print("bwd no dS_T", flush=True)
    _check(inp, "no dS_T", with_dS=False)
    print("bwd no beta", flush=True)
    out, _ = _check(inp, "no beta", with_beta=False)
    # dbeta is still v .* du when asked for
    assert torch.isfinite(out["dbeta"]).all()


def test_strong_decay_and_closed_gates():
    """Hard resets (log_alpha = -inf), very strong decays and alpha = 1 rows inside tiles."""
    inp = _case(1, 160, 2, 128, seed=9)
    la = inp["log_alpha"]
    la[:, 50:60, :, :8] = -30.0
    la[:, 100:120] = 0.0
    la[:, 7::31] = float("-inf")
    print("bwd strong decay", flush=True)
    out, ref = _check(inp, "strong decay")
    assert float(out["dlog_alpha"][:, 7::31].abs().max()) == 0.0


def test_strong_decay_wide_values():
    """The same routes with dv = 256 (eight wavefronts per workgroup in the reverse sweep)."""
    inp = _case(1, 100, 2, 256, seed=19)
    la = inp["log_alpha"]
    la[:, 20:30, :, 5:40] = -25.0
    la[:, 60:70] = 0.0
    la[:, 3::17] = float("-inf")
    print("bwd strong decay dv256", flush=True)
    out, ref = _check(inp, "strong decay dv256")
    assert float(out["dlog_alpha"][:, 3::17].abs().max()) == 0.0


def test_long_sequence_mid_config():
    """Half of the mid configuration (B=2, T=2048, H=8, dv=128): 128 tiles of carried state and cotangent."""
    print("bwd mid-size", flush=True)
    _check(_case(2, 2048, 8, 128, s0=False, seed=21), "mid")


def test_layer_head_shape():
    """The layer's head shape (dv = 256, 16 heads) at T = 1024."""
    print("bwd layer shape", flush=True)
    _check(_case(2, 1024, 16, 256, seed=22), "layer")


@pytest.mark.parametrize("B,T,H,dv,s0", [
    (1, 1000, 2, 256, True),     # four segments of 256 tokens, the last one ragged (232 = 14 * 16 + 8)
    (2, 520, 1, 128, True),      # 9 chunks -> three segments of 192 tokens, the last one 136
    (1, 768, 3, 128, False),     # zero initial state
    (1, 16424, 1, 256, True),    # 257 chunks -> 52 segments of 5 chunks, the last one 2 chunks and 40 tokens
])
def test_sequence_cut_into_segments(B, T, H, dv, s0):
    """Few (batch, head) pairs and a long sequence: the call is cut along the sequence, boundary states and cotangents
    come from the summary passes."""
    print(f"bwd segments B{B} T{T} H{H} dv{dv} s0={s0}", flush=True)
    _check(_case(B, T, H, dv, s0, seed=T + dv + 1), f"segments B{B}T{T}H{H}dv{dv}")


def test_segments_with_weak_decay():
    """Decays near one (a sequence's total decay is about exp(-3)): the states and cotangents handed across the segment
    borders dominate every gradient, so a wrong border term cannot hide behind the decay."""
    print("bwd segments weak decay", flush=True)
    _check(_case(1, 1000, 2, 256, seed=33, gate_mean=-6.0), "segments weak decay")
    print("bwd segments weak decay, 32 segments", flush=True)
    _check(_case(1, 8192, 1, 128, seed=34, gate_mean=-5.0), "segments long")


def test_segments_without_state_cotangent_and_with_resets():
    """Segment route with dS_T = NULL, no value gate, and hard resets / strong decays inside and at segment borders."""
    inp = _case(1, 1024, 2, 256, seed=31)
    la = inp["log_alpha"]
    la[:, 255] = float("-inf")               # the last token of a segment
    la[:, 256, :, :16] = float("-inf")       # the first token of the next one
    la[:, 600:640, :, 8:24] = -20.0
    la[:, 700:760] = 0.0
    print("bwd segments no dS_T", flush=True)
    _check(inp, "segments no dS_T", with_dS=False)
    print("bwd segments no beta", flush=True)
    out, _ = _check(inp, "segments no beta", with_beta=False)
    assert float(out["dlog_alpha"][:, 255].abs().max()) == 0.0


def test_full_size_layer_workload():
    """The layer workload at its full size (B=8, T=4096, H=16, dv=256: 256 workgroups, no cut), in the launch configuration
    bench.py times; the oracle runs all eight sequences and every gradient is compared per sequence."""
    w = wl.LAYER_1P6B
    print("bwd full layer workload: inputs ...", flush=True)
    inp = wl.make_scan_inputs(w)
    rng = np.random.Generator(np.random.PCG64(77))
    inp["d_o"] = torch.from_numpy(rng.standard_normal((w.B, w.T, w.H, w.dv), dtype=np.float32)).to(torch.bfloat16)
    inp["dS_T"] = torch.from_numpy(rng.standard_normal((w.B, w.H, w.dk, w.dv), dtype=np.float32) * np.float32(0.1))
    g = to_dev(inp)
    print("bwd full layer workload: GPU ...", flush=True)
    out = rodimus.rodimus_chunk_scan_bwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], g["d_o"], g["dS_T"])
    torch.cuda.synchronize()
    names = ("dq", "dk", "dv", "dlog_alpha", "dbeta", "dS0")
    for name in names:
        assert torch.isfinite(out[name].float()).all(), name
    for b0 in range(0, w.B, 4):           # four sequences per oracle call: 64 (batch, head) recurrences over the host cores
        print(f"bwd full layer workload: oracle on sequences {b0} .. {b0 + 3} ...", flush=True)
        part = {k: v[b0:b0 + 4].contiguous() for k, v in inp.items()}
        ref = oracle.scan_bwd(part["q"], part["k"], part["v"], part["log_alpha"], part["beta"], part["S0"], part["d_o"], part["dS_T"])
        for b in range(b0, b0 + 4):
            errs = {name: rel_err(out[name][b:b + 1], ref[name][b - b0:b - b0 + 1]) for name in names}
            print(f"   sequence {b}: " + "  ".join(f"{k} {v:.2e}" for k, v in errs.items()), flush=True)
            for name, e in errs.items():
                assert e <= TOL_BF16, (b, name, e)


def test_unsupported_shapes_are_refused():
    # a state that neither kernel family holds: 128 x 256 in fp32 I/O (the token-by-token kernels keep it in LDS)
    x = torch.zeros(1, 4, 1, 128, device="cuda:0")
    v = torch.zeros(1, 4, 1, 256, device="cuda:0")
    with pytest.raises(rodimus.RodimusError) as e:
        rodimus.rodimus_chunk_scan_bwd(x, x, v, x, None, None, v)
    assert e.value.status == 2
