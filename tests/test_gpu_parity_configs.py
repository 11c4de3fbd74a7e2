"""GPU parity at the FULL sizes of the baseline file's configurations, in the launch configuration bench.py times
(needs an MI355X).  The fp64 oracle finishes each of them in seconds on the machine's host cores, so every output
element is compared; the decode configuration is checked on a subset of sequences (sequences are independent, so
the subset check is exact for those sequences)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, gpu_scan, oracle_scan, rel_err, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["layer_1p6b", "long_context"])
def test_full_size_scan_configs(name):
    w = wl.SCAN_WORKLOADS[name]
    print(f"{name}: generating inputs ...", flush=True)
    inp = wl.make_scan_inputs(w)
    assert rodimus.rodimus_chunk_scan_path(w.B, w.T, w.H, w.dk, w.dv, w.chunk, torch.bfloat16) == rodimus.PATH_MFMA
    print(f"{name}: GPU scan ...", flush=True)
    o, S_T = gpu_scan(inp, w.chunk)
    print(f"{name}: oracle ({oracle.threads()} threads) ...", flush=True)
    o_ref, S_ref = oracle_scan(inp)
    eo, es = rel_err(o, o_ref), rel_err(S_T, S_ref)
    print(f"{name}: o rel err {eo:.2e}, S_T rel err {es:.2e}", flush=True)
    assert eo <= TOL_BF16 and es <= TOL_BF16
    # per-(batch, head) check as well: a single bad sequence must not hide behind the global maximum
    go = o.float().cpu().numpy().astype(np.float64)
    for b in range(w.B):
        for h in range(w.H):
            ref = o_ref[b, :, h]
            assert np.abs(go[b, :, h] - ref).max() <= TOL_BF16 * np.abs(ref).max(), (b, h)


def test_decode_config_1000_chained_steps():
    """256 sequences x 16 heads of 64x256 fp32 states, 1000 chained steps on the GPU; the oracle follows 8 of the
    sequences through all 1000 steps."""
    w = wl.DECODE
    d = wl.make_decode_inputs(w)
    sub = [0, 1, 2, 100, 101, 200, 254, 255]
    S = d["S"].to("cuda:0")
    ring = [to_dev(tok) for tok in d["ring"]]
    S_ref = d["S"][sub].double().numpy()
    check_steps = {0, 1, 2, 499, 998, 999}
    print("decode: 1000 chained steps ...", flush=True)
    outs = {}
    for i in range(w.steps):
        t = ring[i % w.ring]
        o = rodimus.rodimus_decode_step(t["q"], t["k"], t["v"], t["log_alpha"], t["beta"], S)
        if i in check_steps:
            outs[i] = o[sub].float().cpu().numpy().astype(np.float64)
    torch.cuda.synchronize()
    print("decode: oracle on the subset ...", flush=True)
    worst = 0.0
    for i in range(w.steps):
        tok = d["ring"][i % w.ring]
        o_ref, S_ref = oracle.step(tok["q"][sub], tok["k"][sub], tok["v"][sub], tok["log_alpha"][sub], tok["beta"][sub], S_ref)
        if i in check_steps:
            e = float(np.abs(outs[i] - o_ref).max() / np.abs(o_ref).max())
            worst = max(worst, e)
            assert e <= TOL_BF16, (i, e)
    es = rel_err(S[sub], S_ref)
    print(f"decode: worst o rel err {worst:.2e}, final S rel err {es:.2e}", flush=True)
    assert es <= 1e-4          # the state never leaves fp32
    assert torch.isfinite(S).all()
