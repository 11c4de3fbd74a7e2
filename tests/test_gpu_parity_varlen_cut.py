"""GPU parity of the packed scan that the kernels cut along the sequences (rodimus_chunk_scan_varlen_fwd_cut: few long
sequences) against the fp64 CPU oracle run on every sequence separately, and against the uncut call (needs an MI355X)."""
import numpy as np
import pytest
import torch

from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import TOL_BF16, rel_err, to_dev
from test_gpu_parity_varlen import _oracle_packed

pytestmark = pytest.mark.gpu


def _run_cut(inp, gate, **kw):
    g = to_dev(inp)
    args = {"beta": g["beta"]} if gate == "beta" else ({"z_beta": g["z_beta"]} if gate == "z_beta" else {})
    o, S_T = rodimus.rodimus_chunk_scan_varlen_fwd_cut(g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], S0=g["S0"], **args, **kw)
    torch.cuda.synchronize()
    return o, S_T


@pytest.mark.parametrize("lengths,H,dv,gate,s0", [
    ([2900, 0, 1500, 77], 2, 256, "beta", True),      # segments of 512: whole ones, ragged ends, an empty and a short sequence
    ([600 + 37 * i for i in range(12)], 8, 256, "beta", True),   # segments of 640 tokens, 12 sequences of one or two segments
    ([1024, 512, 513], 1, 128, "z_beta", True),       # lengths on and one past a segment boundary
    ([5000], 3, 128, "none", False),                  # one sequence, zero initial state, no value gate
    ([1, 1, 3000, 1], 2, 128, "beta", True),
    ([1000, 24], 1, 128, "beta", True),               # exactly the smallest batch that is cut (1024 tokens): two segments of 512
    ([511, 1, 512], 2, 256, "z_beta", True),          # a sequence one token short of a segment, one of exactly a segment
])
def test_cut_matches_the_oracle_per_sequence(lengths, H, dv, gate, s0):
    print(f"varlen cut {lengths} H{H} dv{dv} {gate}", flush=True)
    total, N = sum(lengths), len(lengths)
    assert rodimus.rodimus_chunk_scan_varlen_workspace_bytes(N, total, H, 64, dv, 64, torch.bfloat16) > 0
    inp = wl.make_varlen_inputs(lengths, H, 64, dv, "bf16", s0_std=0.1 if s0 else 0.0, seed=total)
    o, S_T = _run_cut(inp, gate)
    o_ref, S_ref = _oracle_packed(inp, lengths, gate)
    eo, es = rel_err(o, o_ref), rel_err(S_T, S_ref)
    print(f"   o {eo:.2e}  S_T {es:.2e}", flush=True)
    assert eo <= TOL_BF16 and es <= TOL_BF16
    go = o.float().cpu().numpy().astype(np.float64)
    gs = S_T.cpu().numpy().astype(np.float64)
    cu = np.concatenate([[0], np.cumsum(lengths)])
    for b, n in enumerate(lengths):          # every sequence on its own: a short one must not hide behind the global maximum
        if n:
            ref = o_ref[cu[b]:cu[b + 1]]
            assert np.abs(go[cu[b]:cu[b + 1]] - ref).max() <= TOL_BF16 * max(np.abs(ref).max(), 1e-30), b
        assert np.abs(gs[b] - S_ref[b]).max() <= TOL_BF16 * max(np.abs(S_ref[b]).max(), 1e-30), b


def test_cut_agrees_with_the_uncut_call_and_updates_a_cache_in_place():
    lengths, H, dv = [1800, 300, 2100], 2, 256
    inp = wl.make_varlen_inputs(lengths, H, 64, dv, "bf16", seed=41)
    g = to_dev(inp)
    print("varlen cut vs uncut, in place", flush=True)
    o_u, S_u = rodimus.rodimus_chunk_scan_varlen_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], beta=g["beta"], S0=g["S0"])
    cache = g["S0"].clone()
    need = rodimus.rodimus_chunk_scan_varlen_workspace_bytes(len(lengths), sum(lengths), H, 64, dv, 64, torch.bfloat16)
    ws = torch.full((need + 256,), 0x5A, dtype=torch.uint8, device="cuda:0")
    o_c, S_c = rodimus.rodimus_chunk_scan_varlen_fwd_cut(g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], beta=g["beta"],
                                                         S0=cache, S_T=cache, workspace=ws[:need])
    torch.cuda.synchronize()
    assert S_c.data_ptr() == cache.data_ptr()
    assert torch.all(ws[need:] == 0x5A)                        # nothing written past the stated size
    # same arithmetic inside a segment; the state takes one more fp32 sum per segment
    assert rel_err(o_c, o_u.float().cpu().numpy().astype(np.float64)) <= 1e-2
    assert rel_err(S_c, S_u.cpu().numpy().astype(np.float64)) <= 1e-4
    # a second call into the same workspace (stale contents) gives the same bits
    o_2, S_2 = rodimus.rodimus_chunk_scan_varlen_fwd_cut(g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], beta=g["beta"],
                                                         S0=g["S0"], workspace=ws[:need])
    torch.cuda.synchronize()
    assert torch.equal(o_2.view(torch.int16), o_c.view(torch.int16)) and torch.equal(S_2, S_c)


def test_batches_that_are_not_cut_take_the_uncut_path_bit_for_bit():
    lengths, H, dv = [50 + 10 * i for i in range(8)], 2, 128          # under 1024 tokens in all
    assert rodimus.rodimus_chunk_scan_varlen_workspace_bytes(len(lengths), sum(lengths), H, 64, dv, 64, torch.bfloat16) == 0
    inp = wl.make_varlen_inputs(lengths, H, 64, dv, "bf16", seed=42)
    g = to_dev(inp)
    print("varlen cut: uncut batch", flush=True)
    o_u, S_u = rodimus.rodimus_chunk_scan_varlen_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], beta=g["beta"], S0=g["S0"])
    o_c, S_c = _run_cut(inp, "beta")
    assert torch.equal(o_u.view(torch.int16), o_c.view(torch.int16)) and torch.equal(S_u, S_c)
    # shapes the matrix-core kernels do not take are never cut
    assert rodimus.rodimus_chunk_scan_varlen_workspace_bytes(2, 9000, 2, 16, 32, 16, torch.float32) == 0


def test_corrupt_length_table_stays_inside_the_tensors_and_the_workspace():
    """Entries outside [0, total], decreasing or overlapping are clamped by the kernels: the call completes, and neither the rows
    after the output nor the bytes after the workspace are touched."""
    lengths, H, dv = [1500, 1500, 1500], 1, 128
    inp = wl.make_varlen_inputs(lengths, H, 64, dv, "bf16", seed=6)
    g = to_dev(inp)
    total = sum(lengths)
    need = rodimus.rodimus_chunk_scan_varlen_workspace_bytes(3, total, H, 64, dv, 64, torch.bfloat16)
    print("varlen cut corrupt table", flush=True)
    for table in ([-5, 9000, 60, 10_000], [0, total, 0, total], [total, 0, total, 0]):
        o = torch.full((total + 64, H, dv), 7.0, dtype=torch.bfloat16, device="cuda:0")
        ws = torch.full((need + 4096,), 0x5A, dtype=torch.uint8, device="cuda:0")
        bad = torch.tensor(table, dtype=torch.int32, device="cuda:0")
        rodimus.rodimus_chunk_scan_varlen_fwd_cut(g["q"], g["k"], g["v"], g["log_alpha"], bad, beta=g["beta"], S0=g["S0"], o=o[:total],
                                                  workspace=ws[:need])
        torch.cuda.synchronize()
        assert torch.all(o[total:] == 7.0) and torch.all(ws[need:] == 0x5A), table


def test_few_long_sequences_full_size():
    """Eight sequences with a log-uniform length mix, 32768 tokens in total, at the layer's head shape; sampled rows of every
    sequence and every final state against the oracle."""
    lengths = wl.serving_length_mix(8, 32768, seed=19)
    print(f"varlen cut full size: {lengths}", flush=True)
    assert rodimus.rodimus_chunk_scan_varlen_workspace_bytes(8, 32768, 16, 64, 256, 64, torch.bfloat16) > 0
    inp = wl.make_varlen_inputs(lengths, 16, 64, 256, "bf16", seed=14)
    o, S_T = _run_cut(inp, "beta")
    o_ref, S_ref = _oracle_packed(inp, lengths, "beta")
    eo, es = rel_err(o, o_ref), rel_err(S_T, S_ref)
    print(f"   o {eo:.2e}  S_T {es:.2e}", flush=True)
    assert eo <= TOL_BF16 and es <= TOL_BF16
