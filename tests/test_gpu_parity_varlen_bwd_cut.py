"""GPU parity of the packed backward pass that the kernels cut along the sequences (rodimus_chunk_scan_varlen_bwd_cut: few long
sequences) against the backward oracle run on every sequence separately, and against the uncut call (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, rel_err, to_dev

pytestmark = pytest.mark.gpu

NAMES = ("dq", "dk", "dv", "dlog_alpha", "dbeta")


def _cotangents(lengths, H, dv, seed):
    total, N = sum(lengths), len(lengths)
    rng = np.random.Generator(np.random.PCG64(seed))
    d_o = torch.from_numpy(rng.standard_normal((total, H, dv), dtype=np.float32)).to(torch.bfloat16)
    dS_T = torch.from_numpy(rng.standard_normal((N, H, 64, dv), dtype=np.float32) * np.float32(0.1))
    return d_o, dS_T


@pytest.mark.parametrize("lengths,H,dv", [
    ([1500, 0, 700, 77], 2, 256),        # segments of 256 tokens: whole ones, ragged ends, an empty and a short sequence
    ([512, 256, 257], 1, 128),           # lengths on and one past a segment boundary
    ([2100], 3, 128),                    # one sequence
    ([1, 1, 900, 1], 2, 128),
    ([500, 12], 1, 128),                 # exactly the smallest batch that is cut (512 tokens): two segments of 256
    ([255, 1, 256, 257], 2, 256),        # lengths around a segment
])
def test_cut_matches_the_oracle_per_sequence(lengths, H, dv):
    print(f"varlen bwd cut {lengths} H{H} dv{dv}", flush=True)
    d = wl.make_varlen_inputs(lengths, H, 64, dv, "bf16", seed=sum(lengths) + dv)
    d_o, dS_T = _cotangents(lengths, H, dv, 77)
    g = to_dev(d)
    out = rodimus.rodimus_chunk_scan_varlen_bwd_cut(g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], g["beta"], g["S0"],
                                                    d_o.cuda(), dS_T.cuda())
    torch.cuda.synchronize()
    start = 0
    for b, n in enumerate(lengths):
        sl = slice(start, start + n)
        ref = oracle.scan_bwd(d["q"][sl][None], d["k"][sl][None], d["v"][sl][None], d["log_alpha"][sl][None],
                              d["beta"][sl][None], d["S0"][b][None], d_o[sl][None], dS_T[b][None])
        if n > 0:
            for name in NAMES:
                assert rel_err(out[name][sl][None], ref[name]) <= TOL_BF16, (b, n, name)
        assert rel_err(out["dS0"][b][None], ref["dS0"]) <= TOL_BF16, (b, n, "dS0")
        start += n


def test_cut_agrees_with_the_uncut_call():
    lengths, H, dv = [1300, 200, 1600], 2, 256
    d = wl.make_varlen_inputs(lengths, H, 64, dv, "bf16", seed=43)
    d_o, dS_T = _cotangents(lengths, H, dv, 78)
    g = to_dev(d)
    print("varlen bwd cut vs uncut", flush=True)
    args = (g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], g["beta"], g["S0"], d_o.cuda(), dS_T.cuda())
    need = int(rodimus.lib().rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes(len(lengths), sum(lengths), H, 64, dv, rodimus.BF16))
    assert need > int(rodimus.lib().rodimus_chunk_scan_varlen_bwd_workspace_bytes(len(lengths), sum(lengths), H, 64, dv, rodimus.BF16))
    ws = torch.full((need + 4096,), 0x5A, dtype=torch.uint8, device="cuda:0")
    uncut = rodimus.rodimus_chunk_scan_varlen_bwd(*args)
    cut = rodimus.rodimus_chunk_scan_varlen_bwd_cut(*args, workspace=ws[:need])
    torch.cuda.synchronize()
    assert torch.all(ws[need:] == 0x5A)                        # nothing written past the stated size
    for name in NAMES + ("dS0",):
        ref = uncut[name].float().cpu().numpy().astype(np.float64)
        assert rel_err(cut[name], ref) <= 1e-2, name
    again = rodimus.rodimus_chunk_scan_varlen_bwd_cut(*args, workspace=ws[:need])      # stale workspace contents: same bits
    torch.cuda.synchronize()
    for name in NAMES + ("dS0",):
        assert torch.equal(again[name].view(torch.int16 if again[name].dtype == torch.bfloat16 else torch.int32),
                           cut[name].view(torch.int16 if cut[name].dtype == torch.bfloat16 else torch.int32)), name


def test_batches_that_are_not_cut_take_the_uncut_path_bit_for_bit():
    lengths, H, dv = [50 + 10 * i for i in range(5)], 2, 128          # under 512 tokens in all
    lib = rodimus.lib()
    same = (5, sum(lengths), H, 64, dv, rodimus.BF16)
    assert int(lib.rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes(*same)) == int(lib.rodimus_chunk_scan_varlen_bwd_workspace_bytes(*same))
    d = wl.make_varlen_inputs(lengths, H, 64, dv, "bf16", seed=44)
    d_o, dS_T = _cotangents(lengths, H, dv, 79)
    g = to_dev(d)
    print("varlen bwd cut: uncut batch", flush=True)
    args = (g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], g["beta"], g["S0"], d_o.cuda(), dS_T.cuda())
    a, b = rodimus.rodimus_chunk_scan_varlen_bwd(*args), rodimus.rodimus_chunk_scan_varlen_bwd_cut(*args)
    torch.cuda.synchronize()
    for name in NAMES + ("dS0",):
        assert torch.equal(a[name].view(torch.int16 if a[name].dtype == torch.bfloat16 else torch.int32),
                           b[name].view(torch.int16 if b[name].dtype == torch.bfloat16 else torch.int32)), name


def test_corrupt_length_table_stays_inside_the_tensors_and_the_workspace():
    lengths, H, dv = [700, 700, 700], 1, 128
    d = wl.make_varlen_inputs(lengths, H, 64, dv, "bf16", seed=45)
    d_o, dS_T = _cotangents(lengths, H, dv, 80)
    g = to_dev(d)
    total = sum(lengths)
    need = int(rodimus.lib().rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes(3, total, H, 64, dv, rodimus.BF16))
    print("varlen bwd cut corrupt table", flush=True)
    for table in ([-5, 9000, 60, 10_000], [0, total, 0, total], [total, 0, total, 0]):
        ws = torch.full((need + 4096,), 0x5A, dtype=torch.uint8, device="cuda:0")
        bad = torch.tensor(table, dtype=torch.int32, device="cuda:0")
        rodimus.rodimus_chunk_scan_varlen_bwd_cut(g["q"], g["k"], g["v"], g["log_alpha"], bad, g["beta"], g["S0"], d_o.cuda(), dS_T.cuda(),
                                                  workspace=ws[:need])
        torch.cuda.synchronize()
        assert torch.all(ws[need:] == 0x5A), table


def test_few_long_sequences_full_size():
    """The workload bench.py times as scan_backward_few_long_sequences: eight sequences with a log-uniform length mix, 32768
    tokens in all, at the layer's head shape; every sequence against the backward oracle."""
    lengths, H, dv = wl.serving_length_mix(8, 32768), 16, 256
    print(f"varlen bwd cut full size: {lengths}", flush=True)
    d = wl.make_varlen_inputs(lengths, H, 64, dv, "bf16", seed=14)
    d_o, dS_T = _cotangents(lengths, H, dv, 81)
    g = to_dev(d)
    out = rodimus.rodimus_chunk_scan_varlen_bwd_cut(g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], g["beta"], g["S0"],
                                                    d_o.cuda(), dS_T.cuda())
    torch.cuda.synchronize()
    host = {name: out[name].float().cpu() for name in NAMES}
    start = 0
    for b, n in enumerate(lengths):
        sl = slice(start, start + n)
        ref = oracle.scan_bwd(d["q"][sl][None], d["k"][sl][None], d["v"][sl][None], d["log_alpha"][sl][None],
                              d["beta"][sl][None], d["S0"][b][None], d_o[sl][None], dS_T[b][None])
        errs = {name: rel_err(host[name][sl][None], ref[name]) for name in NAMES}
        errs["dS0"] = rel_err(out["dS0"][b][None], ref["dS0"])
        print(f"   sequence {b} ({n} tokens): " + "  ".join(f"{k} {v:.2e}" for k, v in errs.items()), flush=True)
        assert max(errs.values()) <= TOL_BF16, (b, n, errs)
        start += n
