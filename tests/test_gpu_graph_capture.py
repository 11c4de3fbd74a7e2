"""The library's calls can be recorded into a HIP graph (they allocate nothing, do not synchronise and launch on the
caller's stream): a captured decode loop and a captured prefill scan are replayed several times, with eager work and
synchronisations between the replays, and every replay is compared with the eager result (needs an MI355X)."""
import pytest
import torch

from paper_2410_06577_amd import rodimus, workloads as wl
from _parity import to_dev

pytestmark = pytest.mark.gpu


def test_captured_decode_loop_replays_like_eager_steps():
    N, H, dk, dv, steps = 8, 4, 64, 256, 6
    w = wl.DecodeWorkload("g", N=N, H=H, dk=dk, dv=dv, io_dtype="bf16", steps=steps, ring=steps, seed=4)
    d = wl.make_decode_inputs(w)
    ring = [to_dev(tok) for tok in d["ring"]]
    S0 = d["S"].cuda()

    def run_steps(S, outs):
        for i, t in enumerate(ring):
            rodimus.rodimus_decode_step(t["q"], t["k"], t["v"], t["log_alpha"], t["beta"], S, o=outs[i])

    # eager reference
    S_eager = S0.clone()
    o_eager = [torch.empty((N, H, dv), dtype=torch.bfloat16, device="cuda") for _ in range(steps)]
    run_steps(S_eager, o_eager)
    torch.cuda.synchronize()

    # capture (static buffers), after a warm-up launch on the capture stream
    S_graph = S0.clone()
    o_graph = [torch.empty_like(x) for x in o_eager]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run_steps(S_graph, o_graph)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run_steps(S_graph, o_graph)
    for replay in range(3):
        S_graph.copy_(S0)                      # eager work between the replays
        for x in o_graph:
            x.fill_(0)                         # a fill kernel, not a memset node
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(S_graph, S_eager), replay
        for a, b in zip(o_graph, o_eager):
            assert torch.equal(a, b), replay


def test_captured_prefill_scan_replays_like_the_eager_call():
    w = wl.ScanWorkload("g", B=2, T=300, H=4, dk=64, dv=256, chunk=64, io_dtype="bf16", s0_std=0.1, seed=6)
    g = to_dev(wl.make_scan_inputs(w))
    o_eager, S_eager = rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"])
    torch.cuda.synchronize()
    o = torch.empty_like(o_eager)
    S_T = torch.empty_like(S_eager)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], o=o, S_T=S_T)
    for replay in range(3):
        o.fill_(0)
        S_T.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, o_eager) and torch.equal(S_T, S_eager), replay


def test_captured_backward_pass_replays_like_the_eager_call():
    """The backward pass of a call that is cut along the sequence (two summary passes, two chains, sweeps, gate kernel) and
    of the packed forward scan (which ranks the sequence lengths on the device), recorded and replayed."""
    w = wl.ScanWorkload("g", B=1, T=1000, H=2, dk=64, dv=256, chunk=64, io_dtype="bf16", s0_std=0.1, seed=8)
    g = to_dev(wl.make_scan_inputs(w))
    gen = torch.Generator(device="cpu").manual_seed(3)
    d_o = torch.randn((1, 1000, 2, 256), generator=gen).to(torch.bfloat16).cuda()
    dS_T = (0.1 * torch.randn((1, 2, 64, 256), generator=gen)).cuda()
    need = rodimus.lib().rodimus_chunk_scan_bwd_workspace_bytes(1, 1000, 2, 64, 256, rodimus.BF16)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    eager = rodimus.rodimus_chunk_scan_bwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], d_o, dS_T, workspace=ws)
    eager = {k: v.clone() for k, v in eager.items()}
    lengths = [300, 17, 0, 450, 233]
    pk = to_dev(wl.make_varlen_inputs(lengths, 2, 64, 256, "bf16", seed=9))
    o_eager, S_eager = rodimus.rodimus_chunk_scan_varlen_fwd(pk["q"], pk["k"], pk["v"], pk["log_alpha"], pk["cu_seqlens"],
                                                             beta=pk["beta"], S0=pk["S0"])
    torch.cuda.synchronize()
    o = torch.empty_like(o_eager)
    S_T = torch.empty_like(S_eager)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        out = rodimus.rodimus_chunk_scan_bwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], d_o, dS_T, workspace=ws)
        rodimus.rodimus_chunk_scan_varlen_fwd(pk["q"], pk["k"], pk["v"], pk["log_alpha"], pk["cu_seqlens"], beta=pk["beta"],
                                              S0=pk["S0"], o=o, S_T=S_T)
    for replay in range(3):
        for x in out.values():
            x.fill_(0)
        ws.fill_(0)
        o.fill_(0)
        S_T.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, ref in eager.items():
            assert torch.equal(out[name], ref), (replay, name)
        assert torch.equal(o, o_eager) and torch.equal(S_T, S_eager), replay


def test_captured_packed_whole_block_with_the_device_side_cut_replays_like_the_eager_call():
    """A serving prefill in one graph: the whole block over a packed batch, the sequences cut into segments by the kernels
    (summary pass, chain, main pass), the state cache updated in place."""
    lengths, H, dv = [1800, 300, 0, 2100], 2, 256
    total, N = sum(lengths), len(lengths)
    d = wl.make_gated_scan_inputs(1, total, H, 64, dv, "bf16", s0_std=0.0, seed=5)
    g = {k: (None if v is None else v[0].cuda()) for k, v in d.items()}
    gen = torch.Generator(device="cpu").manual_seed(9)
    x_prime = torch.randn((total, H, dv), generator=gen).to(torch.bfloat16).cuda()
    z_gate = torch.randn((total, H, dv), generator=gen).to(torch.bfloat16).cuda()
    d_w = torch.randn((H, dv), generator=gen).cuda()
    cache0 = (0.1 * torch.randn((N, H, 64, dv), generator=gen)).cuda()
    cu = torch.tensor([0, 1800, 2100, 2100, 4200], dtype=torch.int32, device="cuda")
    need = rodimus.rodimus_chunk_scan_varlen_workspace_bytes(N, total, H, 64, dv, 64, torch.bfloat16)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")

    def run(cache, y):
        rodimus.rodimus_chunk_scan_varlen_fwd_gated_block(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], cu, g["z_beta"], cache,
                                                          x_prime=x_prime, d=d_w, z_gate=z_gate, gate_act="silu", o=y, S_T=cache,
                                                          workspace=ws)

    cache_eager, y_eager = cache0.clone(), torch.empty((total, H, dv), dtype=torch.bfloat16, device="cuda")
    run(cache_eager, y_eager)
    torch.cuda.synchronize()
    cache, y = cache0.clone(), torch.empty_like(y_eager)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(cache, y)
    for replay in range(3):
        cache.copy_(cache0)
        y.fill_(0)
        ws.fill_(0x5A)                         # stale workspace contents must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager) and torch.equal(cache, cache_eager), replay
