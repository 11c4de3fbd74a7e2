#!/usr/bin/env python3
"""Benchmark of the Rodimus DDTS hot path on one MI355X.  Prints ONE JSON line.

A "step" is one forward chunk scan (rodimus_chunk_scan_fwd) over the 1.6B-class layer batch
(B=8, T=4096, H=16, dk=64, dv=256, chunk=64; bf16 q/k/v/o, fp32 gates and state, non-zero S0,
S_T returned), inputs resident in HBM.  `value` is tokens/s of that scan (tokens = B*T positions,
all heads).  The decode leg then times 1000 chained rodimus_decode_step launches over 256
sequences x 16 heads of 64x256 fp32 states and is reported in the `decode` object of the same
line, with its own roofline.  `cpu_baseline` is the fp64 CPU oracle timed on this machine's host
cores on the same scan workload (it finishes in seconds; it also serves as a parity check of the
whole GPU result).

Roofline figures: `achieved` = algorithmic bytes per launch / mean launch duration from HIP events
on the launch stream.  Algorithmic bytes per (token, head): q 2dk + k 2dk + log_alpha 4dk + v 2dv +
beta 4dv + o 2dv = 2560 B at dk=64, dv=256, plus S0 read and S_T written once per (batch, head).
Decode: S read + S written (2*4*dk*dv B per state) plus the token vectors and o.
"""
import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, vendor figure

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (scaled by a plain copy kernel);
# taken from the summaries under profiles/ (scan_mfma_kernel_layer_1p6b.md, decode_step_kernel_256x16.md).
MEASURED_TRAFFIC_BYTES = {"scan_layer_1p6b": 1384.5e6, "decode_256x16": 547.6e6, "decode_512x16": 1094.8e6}   # profiles/*.md


def warm_up(step, launches, min_seconds=0.08):
    """`launches` untimed launches, and more until `min_seconds` of back-to-back GPU work have passed: after an idle
    phase (input generation on the host) the first ~30 ms of launches run up to 25 % slower while the GPU clocks ramp."""
    t0 = time.perf_counter()
    done = 0
    while done < launches or time.perf_counter() - t0 < min_seconds:
        for _ in range(10 if done >= launches else min(10, launches - done)):
            step()
            done += 1
        torch.cuda.synchronize()
    return done


def bench_scan(w, steps, warmup, rodimus, wl, dev, zbeta=False):
    inp = wl.make_scan_inputs(w)
    g = {k: (None if v is None else v.to(dev)) for k, v in inp.items()}
    o = torch.empty((w.B, w.T, w.H, w.dv), dtype=torch.bfloat16, device=dev)
    S_T = torch.empty((w.B, w.H, w.dk, w.dv), dtype=torch.float32, device=dev)
    need = rodimus.rodimus_chunk_scan_workspace_bytes(w.B, w.T, w.H, w.dk, w.dv, w.chunk, torch.bfloat16)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)

    def step():
        if zbeta:      # value gate as bf16 pre-activation, sigmoid inside the kernel
            rodimus.rodimus_chunk_scan_fwd_zbeta(g["q"], g["k"], g["v"], g["log_alpha"], g["z_beta"], g["S0"],
                                                 chunk=w.chunk, o=o, S_T=S_T, workspace=ws)
        else:
            rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"],
                                           chunk=w.chunk, o=o, S_T=S_T, workspace=ws)

    # `warmup` untimed launches as asked, and more until the clocks have settled (see warm_up): with a handful of warm-up
    # launches alone the timed region would still lie in the clock ramp and read up to 25 % slow
    settle = warm_up(step, warmup, min_seconds=0.15)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        step()
    stop.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    launch_ms = start.elapsed_time(stop) / steps      # HIP events on the launch stream around the K back-to-back launches
    # afterwards (outside the timed region): single launches between their own pairs of events, for the median and the minimum
    n_single = min(steps, 50)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_single)]
    for a, b in pairs:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    singles = sorted(a.elapsed_time(b) for a, b in pairs)

    th = w.token_heads
    state_bytes = w.B * w.H * w.dk * w.dv * 4
    algo_bytes = th * (8 * w.dk + (6 if zbeta else 8) * w.dv) + state_bytes * ((1 if g["S0"] is not None else 0) + 1)
    flops_causal = th * 2 * (2 * w.dk * w.dv + w.chunk * (w.dk + w.dv) // 2)
    flops_dense = th * 2 * (2 * w.dk * w.dv + w.chunk * (w.dk + w.dv))
    res = {
        "wall_s": wall, "ms_per_step": wall / steps * 1e3, "launch_ms": launch_ms,
        "tokens_per_s": w.tokens * steps / wall,
        "algo_bytes": algo_bytes, "gbs": algo_bytes / (launch_ms * 1e-3) / 1e9,
        "tflops_causal": flops_causal / (launch_ms * 1e-3) / 1e12,
        "tflops_dense_tiles": flops_dense / (launch_ms * 1e-3) / 1e12,
        "path": rodimus.rodimus_chunk_scan_path(w.B, w.T, w.H, w.dk, w.dv, w.chunk, torch.bfloat16),
        "single_launch_ms": {"median": singles[len(singles) // 2], "min": singles[0], "launches": n_single} if singles else None,
        "settle_launches": settle,
    }
    return res, inp, o, S_T


def bench_scan_outputs(w, inp, rodimus, dev):
    """One untimed scan of the given CPU inputs; returns (o, S_T) for the parity check."""
    g = {k: (None if v is None else v.to(dev)) for k, v in inp.items()}
    o, S_T = rodimus.rodimus_chunk_scan_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], chunk=w.chunk)
    torch.cuda.synchronize()
    return o, S_T


def bench_decode(w, rodimus, wl, dev, warmup=100):
    d = wl.make_decode_inputs(w)
    S = d["S"].to(dev)
    ring = [{k: v.to(dev) for k, v in tok.items()} for tok in d["ring"]]
    o = torch.empty((w.N, w.H, w.dv), dtype=torch.bfloat16, device=dev)

    def step(i):
        t = ring[i % len(ring)]
        rodimus.rodimus_decode_step(t["q"], t["k"], t["v"], t["log_alpha"], t["beta"], S, o=o)

    count = [0]

    def warm_step():
        step(count[0])
        count[0] += 1

    warm_up(warm_step, warmup)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    a.record()
    for i in range(w.steps):
        step(i)
    b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    launch_ms = a.elapsed_time(b) / w.steps
    states = w.N * w.H
    algo_bytes = states * (2 * 4 * w.dk * w.dv + 2 * (2 * w.dk) + 4 * w.dk + 2 * w.dv + 4 * w.dv + 2 * w.dv)
    finite = bool(torch.isfinite(S).all().item())
    return {"wall_s": wall, "launch_ms": launch_ms, "algo_bytes": algo_bytes,
            "gbs": algo_bytes / (launch_ms * 1e-3) / 1e9, "steps_per_s": w.steps / wall, "finite": finite}


def decode_cpu_baseline(w, wl, steps=10):
    """The step oracle over all sequences of the decode workload for a few chained steps, on the host cores."""
    import oracle
    d = wl.make_decode_inputs(w)
    S = d["S"].double().numpy()
    t0 = time.perf_counter()
    for i in range(steps):
        tok = d["ring"][i % len(d["ring"])]
        _, S = oracle.step(tok["q"], tok["k"], tok["v"], tok["log_alpha"], tok["beta"], S)
    dt = (time.perf_counter() - t0) / steps
    states = w.N * w.H
    algo_bytes = states * (2 * 4 * w.dk * w.dv + 2 * (2 * w.dk) + 4 * w.dk + 2 * w.dv + 4 * w.dv + 2 * w.dv)
    return {"value": algo_bytes / dt / 1e9, "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"{steps} chained steps over all {w.N} sequences (fp64 state; GB/s counted on the GPU step's algorithmic bytes), "
                      f"{dt * 1e3:.0f} ms per step"}


def bench_decode_small(rodimus, wl, dev, H=16, dk=64, dv=256, chained=64, reps=20):
    """Latency of the decode step at serving batch sizes where the launch, not the bandwidth, is the cost: `chained` steps
    issued one by one from Python, and the same steps recorded once into a HIP graph and replayed."""
    out = {}
    for N in (1, 8, 32):
        w = wl.DecodeWorkload("small", N=N, H=H, dk=dk, dv=dv, io_dtype="bf16", steps=chained, ring=8, seed=5)
        d = wl.make_decode_inputs(w)
        S = d["S"].to(dev)
        ring = [{k: v.to(dev) for k, v in tok.items()} for tok in d["ring"]]
        o = torch.empty((N, H, dv), dtype=torch.bfloat16, device=dev)

        def run():
            for i in range(chained):
                t = ring[i % len(ring)]
                rodimus.rodimus_decode_step(t["q"], t["k"], t["v"], t["log_alpha"], t["beta"], S, o=o)

        run()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        for _ in range(reps):
            run()
        torch.cuda.synchronize()
        eager_us = (time.perf_counter() - t0) / (reps * chained) * 1e6
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run()
        graph.replay()
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            graph.replay()
        b.record()
        torch.cuda.synchronize()
        graph_us = a.elapsed_time(b) / (reps * chained) * 1e3
        out[f"{N}_sequences"] = {"us_per_step_eager": eager_us, "us_per_step_hip_graph": graph_us,
                                 "state_bytes": N * H * dk * dv * 4}
    out["note"] = f"{chained} chained steps; eager = ctypes call per step from Python (wall clock), graph = one replay per {chained} steps"
    return out


def bench_gates(w, rodimus, wl, dev, steps=50, warmup=20):
    """DDTS gate front-end over the token-heads of the scan workload (pre-activations -> log_alpha, beta, q, k)."""
    d = wl.make_ddts_preactivations((w.B, w.T, w.H), w.dk, w.dv, "bf16", seed=9)
    g = {k: v.to(dev) for k, v in d.items()}
    la = torch.empty((w.B, w.T, w.H, w.dk), dtype=torch.float32, device=dev)
    beta = torch.empty((w.B, w.T, w.H, w.dv), dtype=torch.float32, device=dev)
    qo, ko = torch.empty_like(g["q"]), torch.empty_like(g["k"])

    def step():
        rodimus.rodimus_ddts_gates(g["z_g"], g["z_tau"], g["z_beta"], g["q"], g["k"], log_alpha=la, beta=beta, q_out=qo, k_out=ko)

    warm_up(step, warmup)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        step()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / steps
    # key side alone (what remains of this pass when the scan takes the value gate as a pre-activation)
    a.record()
    for _ in range(steps):
        rodimus.rodimus_ddts_gates(g["z_g"], g["z_tau"], None, g["q"], g["k"], log_alpha=la, q_out=qo, k_out=ko)
    b.record()
    torch.cuda.synchronize()
    ms_key = a.elapsed_time(b) / steps
    th = w.token_heads
    algo = th * (4 * 2 * w.dk + 2 * w.dv + 4 * w.dk + 4 * w.dv + 2 * 2 * w.dk)    # 4 bf16 key-side inputs, z_beta; log_alpha, beta, q, k out
    algo_key = th * (4 * 2 * w.dk + 4 * w.dk + 2 * 2 * w.dk)
    return {"ms_per_call": ms, "algorithmic_bytes": algo, "GB_per_s": algo / (ms * 1e-3) / 1e9,
            "hbm_frac": algo / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "token_heads_per_s": th / (ms * 1e-3),
            "key_side_only": {"ms_per_call": ms_key, "algorithmic_bytes": algo_key,
                              "GB_per_s": algo_key / (ms_key * 1e-3) / 1e9}}


def bench_gated_scan(w, rodimus, wl, dev, steps, warmup):
    """The layer scan with the whole gate front-end fused in (rodimus_chunk_scan_fwd_gated), beside the two-call
    pipeline it replaces (key-side rodimus_ddts_gates, then rodimus_chunk_scan_fwd_zbeta) on the same inputs."""
    d = wl.make_gated_scan_inputs(w.B, w.T, w.H, w.dk, w.dv, "bf16", seed=17)
    g = {k: (None if v is None else v.to(dev)) for k, v in d.items()}
    o = torch.empty((w.B, w.T, w.H, w.dv), dtype=torch.bfloat16, device=dev)
    S_T = torch.empty((w.B, w.H, w.dk, w.dv), dtype=torch.float32, device=dev)
    la = torch.empty((w.B, w.T, w.H, w.dk), dtype=torch.float32, device=dev)
    qo, ko = torch.empty_like(g["q"]), torch.empty_like(g["k"])

    def fused():
        rodimus.rodimus_chunk_scan_fwd_gated(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["z_beta"], g["S0"], chunk=w.chunk,
                                             o=o, S_T=S_T)

    def two_calls():
        rodimus.rodimus_ddts_gates(g["z_g"], g["z_tau"], None, g["q"], g["k"], log_alpha=la, q_out=qo, k_out=ko)
        rodimus.rodimus_chunk_scan_fwd_zbeta(qo, ko, g["v"], la, g["z_beta"], g["S0"], chunk=w.chunk, o=o, S_T=S_T)

    def timed(f):
        warm_up(f, warmup)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            f()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / steps

    ms, ms_pipe = timed(fused), timed(two_calls)
    th = w.token_heads
    state_bytes = w.B * w.H * w.dk * w.dv * 4
    algo = th * (4 * 2 * w.dk + 3 * 2 * w.dv) + 2 * state_bytes       # q, k, z_g, z_tau; v, z_beta, o; S0 and S_T
    return {"entry_point": "rodimus_chunk_scan_fwd_gated", "workload": "layer_1p6b, every gate as bf16 pre-activation, raw q and k",
            "ms_per_step": ms, "tokens_per_s": w.tokens / (ms * 1e-3), "algorithmic_bytes": algo,
            "GB_per_s": algo / (ms * 1e-3) / 1e9, "hbm_frac": algo / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "two_call_pipeline_ms": ms_pipe}


def bench_block_scan(w, rodimus, wl, dev, steps, warmup):
    """The layer scan with the block's output stage fused in (rodimus_chunk_scan_fwd_block): feed-through d .* x' and the SiLU
    output gate applied where the outputs leave the kernel, o written once."""
    import numpy as np
    inp = wl.make_scan_inputs(w)
    g = {k: (None if v is None else v.to(dev)) for k, v in inp.items()}
    rng = np.random.Generator(np.random.PCG64(21))
    shape = (w.B, w.T, w.H, w.dv)
    x_prime = torch.from_numpy(rng.standard_normal(shape, dtype=np.float32)).to(torch.bfloat16).to(dev)
    z_gate = torch.from_numpy(rng.standard_normal(shape, dtype=np.float32)).to(torch.bfloat16).to(dev)
    d = torch.from_numpy(rng.standard_normal((w.H, w.dv), dtype=np.float32)).to(dev)
    o = torch.empty(shape, dtype=torch.bfloat16, device=dev)
    S_T = torch.empty((w.B, w.H, w.dk, w.dv), dtype=torch.float32, device=dev)

    def step():
        rodimus.rodimus_chunk_scan_fwd_block(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], x_prime=x_prime, d=d,
                                             z_gate=z_gate, gate_act="silu", chunk=w.chunk, o=o, S_T=S_T)

    warm_up(step, warmup)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        step()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / steps
    th = w.token_heads
    algo = th * (8 * w.dk + 8 * w.dv + 2 * 2 * w.dv) + 2 * w.B * w.H * w.dk * w.dv * 4      # the scan's bytes + x' and z_gate
    return {"entry_point": "rodimus_chunk_scan_fwd_block", "workload": "layer_1p6b + x' and z_gate (bf16), d fp32, SiLU gate",
            "launches_per_call": 1, "ms_per_step": ms, "tokens_per_s": w.tokens / (ms * 1e-3), "algorithmic_bytes": algo,
            "GB_per_s": algo / (ms * 1e-3) / 1e9, "hbm_frac": algo / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}


def bench_whole_block_scan(w, rodimus, wl, dev, steps, warmup):
    """The layer scan with both ends of the block fused in (rodimus_chunk_scan_fwd_gated_block): every gate taken as a bf16
    pre-activation on the way in, feed-through and SiLU output gate on the way out; one launch."""
    import numpy as np
    d = wl.make_gated_scan_inputs(w.B, w.T, w.H, w.dk, w.dv, "bf16", seed=17)
    g = {k: (None if v is None else v.to(dev)) for k, v in d.items()}
    rng = np.random.Generator(np.random.PCG64(21))
    shape = (w.B, w.T, w.H, w.dv)
    x_prime = torch.from_numpy(rng.standard_normal(shape, dtype=np.float32)).to(torch.bfloat16).to(dev)
    z_gate = torch.from_numpy(rng.standard_normal(shape, dtype=np.float32)).to(torch.bfloat16).to(dev)
    dw = torch.from_numpy(rng.standard_normal((w.H, w.dv), dtype=np.float32)).to(dev)
    o = torch.empty(shape, dtype=torch.bfloat16, device=dev)
    S_T = torch.empty((w.B, w.H, w.dk, w.dv), dtype=torch.float32, device=dev)

    def step():
        rodimus.rodimus_chunk_scan_fwd_gated_block(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["z_beta"], g["S0"],
                                                   x_prime=x_prime, d=dw, z_gate=z_gate, gate_act="silu", chunk=w.chunk, o=o, S_T=S_T)

    warm_up(step, warmup)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        step()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / steps
    # q, k, z_g, z_tau; v, z_beta, x', z_gate, o; S0 and S_T
    algo = w.token_heads * (4 * 2 * w.dk + 5 * 2 * w.dv) + 2 * w.B * w.H * w.dk * w.dv * 4
    return {"entry_point": "rodimus_chunk_scan_fwd_gated_block",
            "workload": "layer_1p6b, every gate as bf16 pre-activation, raw q and k, x' and z_gate (bf16), d fp32, SiLU gate",
            "launches_per_call": 1, "ms_per_step": ms, "tokens_per_s": w.tokens / (ms * 1e-3), "algorithmic_bytes": algo,
            "GB_per_s": algo / (ms * 1e-3) / 1e9, "hbm_frac": algo / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}


def bench_stream_probe(rodimus, dev, steps=20):
    """What the memory system of this GPU gives a kernel that only streams (rodimus_hbm_stream_probe): four 16-byte units
    read per unit written, the mix of the layer scan (2048 B read and 512 B written per token and head; 1 GiB read, 256 MiB
    written per launch), and one read per write, the mix and the footprint of the decode step over 512 sequences (512 MiB
    each way).  Best of a few grid sizes each."""
    out = {}
    for name, reads, mib in (("four_reads_per_write", 4, 256), ("one_read_per_write", 1, 512)):
        dst = torch.empty(mib << 20, dtype=torch.uint8, device=dev)
        src = torch.ones(reads * dst.numel(), dtype=torch.uint8, device=dev)
        best, best_wgs = None, None
        for wgs in (256, 512, 1024, 16384, 65536, 262144):
            def step():
                rodimus.rodimus_hbm_stream_probe(src, dst, reads, wgs)
            warm_up(step, 5)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(steps):
                step()
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b) / steps
            if best is None or ms < best:
                best, best_wgs = ms, wgs
        gbs = (reads + 1) * dst.numel() / (best * 1e-3) / 1e9
        out[name] = {"GB_per_s": gbs, "hbm_frac": gbs / HBM_PEAK_GBS, "ms": best, "workgroups": best_wgs,
                     "MiB_written": mib, "MiB_read": reads * mib}
        del src, dst
    return out


def bench_short_conv(w, rodimus, wl, dev, steps=50, warmup=20, width=4):
    """The block's ShortConv over the layer workload's tokens: C = H * dv channels, width 4, SiLU, bf16 I/O."""
    C = w.H * w.dv
    d = wl.make_short_conv_inputs(w.B, w.T, C, width, "bf16", seed=15)
    g = {k: v.to(dev) for k, v in d.items()}
    y = torch.empty_like(g["x"])
    st = torch.empty_like(g["state"])

    def step():
        rodimus.rodimus_short_conv_fwd(g["x"], g["w"], g["bias"], g["state"], y=y, state_out=st)

    warm_up(step, warmup)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        step()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / steps
    algo = 2 * 2 * w.B * w.T * C            # x read once, y written once, bf16
    return {"entry_point": "rodimus_short_conv_fwd", "workload": f"B={w.B} T={w.T} C={C} W={width} SiLU bf16",
            "ms_per_call": ms, "algorithmic_bytes": algo, "GB_per_s": algo / (ms * 1e-3) / 1e9,
            "hbm_frac": algo / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "tokens_per_s": w.B * w.T / (ms * 1e-3)}


def bench_varlen(w, rodimus, wl, dev, steps, warmup, n_seq=64, longest_first=False, cut=False):
    """Packed variable-length prefill: n_seq sequences with a log-uniform length mix and the token count of the layer
    workload (rodimus_chunk_scan_varlen_fwd, states written to a cache; with `cut` rodimus_chunk_scan_varlen_fwd_cut, whose
    kernels cut the sequences into segments that run side by side)."""
    lengths = wl.serving_length_mix(n_seq, w.B * w.T)
    if longest_first:       # workgroups start in sequence order: longest first is the better schedule
        lengths = sorted(lengths, reverse=True)
    d = wl.make_varlen_inputs(lengths, w.H, w.dk, w.dv, "bf16", seed=14)
    g = {k: (None if v is None else v.to(dev)) for k, v in d.items()}
    o = torch.empty((w.B * w.T, w.H, w.dv), dtype=torch.bfloat16, device=dev)
    S_T = torch.empty((n_seq, w.H, w.dk, w.dv), dtype=torch.float32, device=dev)

    need = rodimus.rodimus_chunk_scan_varlen_workspace_bytes(n_seq, w.B * w.T, w.H, w.dk, w.dv, w.chunk, torch.bfloat16) if cut else 0
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)

    def step():
        if cut:
            rodimus.rodimus_chunk_scan_varlen_fwd_cut(g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], beta=g["beta"],
                                                      S0=g["S0"], o=o, S_T=S_T, workspace=ws)
        else:
            rodimus.rodimus_chunk_scan_varlen_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], beta=g["beta"],
                                                  S0=g["S0"], o=o, S_T=S_T)

    warm_up(step, warmup)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        step()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / steps
    algo = w.token_heads * (8 * w.dk + 8 * w.dv) + 2 * n_seq * w.H * w.dk * w.dv * 4
    return {"entry_point": "rodimus_chunk_scan_varlen_fwd_cut" if cut else "rodimus_chunk_scan_varlen_fwd",
            "workload": f"{n_seq} sequences, lengths {min(lengths)}..{max(lengths)} (log-uniform mix), {w.B * w.T} tokens, "
                        f"H={w.H} dk={w.dk} dv={w.dv}",
            "ms_per_step": ms, "tokens_per_s": w.B * w.T / (ms * 1e-3), "GB_per_s": algo / (ms * 1e-3) / 1e9,
            "hbm_frac": algo / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}


def bench_varlen_whole_block(w, rodimus, wl, dev, steps, warmup, n_seq=64):
    """Packed variable-length prefill of the whole block in one launch (rodimus_chunk_scan_varlen_fwd_gated_block): the length mix
    of bench_varlen, every gate as a bf16 pre-activation, raw q and k, feed-through and SiLU output gate."""
    import numpy as np
    lengths = wl.serving_length_mix(n_seq, w.B * w.T)
    total = w.B * w.T
    d = wl.make_gated_scan_inputs(1, total, w.H, w.dk, w.dv, "bf16", s0_std=0.0, seed=17)
    g = {k: (None if v is None else v[0].to(dev)) for k, v in d.items()}
    rng = np.random.Generator(np.random.PCG64(21))
    shape = (total, w.H, w.dv)
    x_prime = torch.from_numpy(rng.standard_normal(shape, dtype=np.float32)).to(torch.bfloat16).to(dev)
    z_gate = torch.from_numpy(rng.standard_normal(shape, dtype=np.float32)).to(torch.bfloat16).to(dev)
    dw = torch.from_numpy(rng.standard_normal((w.H, w.dv), dtype=np.float32)).to(dev)
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lengths)]), dtype=torch.int32, device=dev)
    cache = (0.1 * torch.randn((n_seq, w.H, w.dk, w.dv), generator=torch.Generator().manual_seed(3))).to(dev)
    o = torch.empty(shape, dtype=torch.bfloat16, device=dev)
    S_T = torch.empty_like(cache)

    def step():
        rodimus.rodimus_chunk_scan_varlen_fwd_gated_block(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], cu, g["z_beta"], cache,
                                                          x_prime=x_prime, d=dw, z_gate=z_gate, gate_act="silu", o=o, S_T=S_T)

    warm_up(step, warmup)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        step()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / steps
    algo = w.token_heads * (4 * 2 * w.dk + 5 * 2 * w.dv) + 2 * n_seq * w.H * w.dk * w.dv * 4
    return {"entry_point": "rodimus_chunk_scan_varlen_fwd_gated_block",
            "workload": f"{n_seq} sequences, lengths {min(lengths)}..{max(lengths)} (log-uniform mix), {total} tokens, "
                        f"H={w.H} dk={w.dk} dv={w.dv}, all gates as pre-activations, feed-through and SiLU gate",
            "launches_per_call": 1, "ms_per_step": ms, "tokens_per_s": total / (ms * 1e-3), "algorithmic_bytes": algo,
            "GB_per_s": algo / (ms * 1e-3) / 1e9, "hbm_frac": algo / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}


def bench_backward(w, rodimus, wl, dev, steps, warmup, zbeta=False):
    """Backward pass of the scan over the layer workload (rodimus_chunk_scan_bwd: dq, dk, dv, dlog_alpha, dbeta, dS0; with
    zbeta the form that reads the value gate's bf16 pre-activation and writes its cotangent, rodimus_chunk_scan_bwd_zbeta)."""
    inp = wl.make_scan_inputs(w)
    g = {k: (None if v is None else v.to(dev)) for k, v in inp.items()}
    gen = torch.Generator(device="cpu").manual_seed(17)
    d_o = torch.randn((w.B, w.T, w.H, w.dv), generator=gen).to(torch.bfloat16).to(dev)
    dS_T = (0.1 * torch.randn((w.B, w.H, w.dk, w.dv), generator=gen)).to(dev)
    need = rodimus.lib().rodimus_chunk_scan_bwd_workspace_bytes(w.B, w.T, w.H, w.dk, w.dv, rodimus.BF16)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    out = {}

    def step():
        if zbeta:
            out.update(rodimus.rodimus_chunk_scan_bwd_zbeta(g["q"], g["k"], g["v"], g["log_alpha"], g["z_beta"], g["S0"], d_o, dS_T,
                                                            workspace=ws))
        else:
            out.update(rodimus.rodimus_chunk_scan_bwd(g["q"], g["k"], g["v"], g["log_alpha"], g["beta"], g["S0"], d_o, dS_T,
                                                      workspace=ws))

    warm_up(step, min(warmup, 20), min_seconds=0.2)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n = max(5, steps // 10)
    a.record()
    for _ in range(n):
        step()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / n
    th = w.token_heads
    # per token-head: forward sweep reads q,k,log_alpha,v,beta,do and writes dq and q.*dq; reverse sweep reads the six
    # inputs again and writes dk, k.*dk, dv, dbeta; the gate kernel reads q.*dq, k.*dk, log_alpha and writes dlog_alpha
    gate = 2 if zbeta else 4                      # bytes per element of the value gate and of its cotangent
    inputs = 2 * w.dk * 2 + 4 * w.dk + 2 * w.dv + gate * w.dv + 2 * w.dv
    algo = th * (2 * inputs + (2 * w.dk + 4 * w.dk) + (2 * w.dk + 4 * w.dk + 2 * w.dv + gate * w.dv) + (3 * 4 * w.dk + 4 * w.dk))
    flops = th * 2 * (4 * w.dk * w.dv + 2 * 16 * w.dv + 2 * 16 * w.dk) * 2    # state products + tile-local products, both sweeps
    return {"entry_point": "rodimus_chunk_scan_bwd_zbeta" if zbeta else "rodimus_chunk_scan_bwd", "ms_per_step": ms, "tokens_per_s": w.tokens / (ms * 1e-3),
            "algorithmic_bytes": algo, "GB_per_s": algo / (ms * 1e-3) / 1e9, "hbm_frac": algo / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "tflops": flops / (ms * 1e-3) / 1e12, "finite": bool(torch.isfinite(out["dlog_alpha"]).all().item())}


def bench_backward_few_long(w, rodimus, wl, dev, steps, warmup, n_seq=8):
    """Backward pass over a packed batch of few long sequences (the length mix of serving_prefill_few_long_sequences): one
    workgroup pair per (sequence, head) (rodimus_chunk_scan_varlen_bwd) against the kernels cutting the sequences into segments
    (rodimus_chunk_scan_varlen_bwd_cut)."""
    lengths = wl.serving_length_mix(n_seq, w.B * w.T)
    total = w.B * w.T
    d = wl.make_varlen_inputs(lengths, w.H, w.dk, w.dv, "bf16", seed=14)
    g = {k: (None if v is None else v.to(dev)) for k, v in d.items()}
    gen = torch.Generator(device="cpu").manual_seed(23)
    d_o = torch.randn((total, w.H, w.dv), generator=gen).to(torch.bfloat16).to(dev)
    dS_T = (0.1 * torch.randn((n_seq, w.H, w.dk, w.dv), generator=gen)).to(dev)
    lib = rodimus.lib()
    need = max(int(lib.rodimus_chunk_scan_varlen_bwd_workspace_bytes(n_seq, total, w.H, w.dk, w.dv, rodimus.BF16)),
               int(lib.rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes(n_seq, total, w.H, w.dk, w.dv, rodimus.BF16)))
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    args = (g["q"], g["k"], g["v"], g["log_alpha"], g["cu_seqlens"], g["beta"], g["S0"], d_o, dS_T)
    out, res = {}, {}
    for name, fn in (("uncut", rodimus.rodimus_chunk_scan_varlen_bwd), ("cut", rodimus.rodimus_chunk_scan_varlen_bwd_cut)):
        def step():
            out.update(fn(*args, workspace=ws))
        warm_up(step, 3, min_seconds=0.2)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n = max(3, steps // 20)
        a.record()
        for _ in range(n):
            step()
        b.record()
        torch.cuda.synchronize()
        res[name] = a.elapsed_time(b) / n
    return {"entry_point": "rodimus_chunk_scan_varlen_bwd_cut",
            "workload": f"{n_seq} sequences, lengths {min(lengths)}..{max(lengths)} (log-uniform mix), {total} tokens, "
                        f"H={w.H} dk={w.dk} dv={w.dv}",
            "ms_per_step": res["cut"], "uncut_ms_per_step": res["uncut"], "tokens_per_s": total / (res["cut"] * 1e-3),
            "finite": bool(torch.isfinite(out["dlog_alpha"]).all().item())}


def bench_backward_gated(w, rodimus, wl, dev, steps, warmup):
    """Backward pass of the gated scan over the layer workload (rodimus_chunk_scan_bwd_gated: cotangents of the raw q, k, v and
    of the three pre-activations): key-side gate pass, backward of the scan, backward of the gate pass."""
    d = wl.make_gated_scan_inputs(w.B, w.T, w.H, w.dk, w.dv, "bf16", seed=17)
    g = {k: (None if v is None else v.to(dev)) for k, v in d.items()}
    gen = torch.Generator(device="cpu").manual_seed(19)
    d_o = torch.randn((w.B, w.T, w.H, w.dv), generator=gen).to(torch.bfloat16).to(dev)
    dS_T = (0.1 * torch.randn((w.B, w.H, w.dk, w.dv), generator=gen)).to(dev)
    need = int(rodimus.lib().rodimus_chunk_scan_bwd_gated_workspace_bytes(w.B, w.T, w.H, w.dk, w.dv, rodimus.BF16))
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    out = {}

    def step():
        out.update(rodimus.rodimus_chunk_scan_bwd_gated(g["q"], g["k"], g["v"], g["z_g"], g["z_tau"], g["z_beta"], g["S0"], d_o, dS_T,
                                                        workspace=ws))

    warm_up(step, min(warmup, 20), min_seconds=0.2)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n = max(5, steps // 10)
    a.record()
    for _ in range(n):
        step()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / n
    return {"entry_point": "rodimus_chunk_scan_bwd_gated", "ms_per_step": ms, "tokens_per_s": w.tokens / (ms * 1e-3),
            "workspace_bytes": need, "finite": bool(torch.isfinite(out["dz_g"].float()).all().item())}


def cpu_baseline(w, inp, o_gpu, S_gpu):
    """fp64 oracle on the scan workload, timed on the host cores; also the parity check of the GPU result."""
    import numpy as np
    import oracle
    t0 = time.perf_counter()
    o_ref, S_ref = oracle.scan(inp["q"], inp["k"], inp["v"], inp["log_alpha"], inp["beta"], inp["S0"])
    dt = time.perf_counter() - t0

    def rel(got, ref):
        got = got.detach().cpu().double().numpy()
        return float(np.abs(got - ref).max() / np.abs(ref).max())

    # one (batch, head) of the same workload: the oracle parallelises over (batch, head), so this runs on one thread
    one = {k: (None if v is None else v[:1, :, :1].contiguous()) for k, v in inp.items() if k in ("q", "k", "v", "log_alpha", "beta")}
    s0 = None if inp["S0"] is None else inp["S0"][:1, :1].contiguous()
    t1 = time.perf_counter()
    oracle.scan(one["q"], one["k"], one["v"], one["log_alpha"], one["beta"], s0)
    dt1 = time.perf_counter() - t1
    return {
        "value": w.tokens / dt, "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
        "sample": f"the whole scan workload once (B={w.B}, T={w.T}, H={w.H}, dk={w.dk}, dv={w.dv}), fp64 sequential "
                  f"recurrence, OpenMP over (batch, head), {dt:.2f} s",
        "seconds": dt,
        "single_thread": {"value": w.T / w.H / dt1, "unit": "tokens/s", "cores": 1,
                          "sample": f"one (batch, head) of the workload ({w.T} token-heads), {dt1:.2f} s; tokens/s = token-heads/s / H"},
    }, {"o_rel_err": rel(o_gpu, o_ref), "S_T_rel_err": rel(S_gpu, S_ref), "tolerance": 2e-2}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=200,
                    help="untimed launches before the timed ones (at least this many; every leg goes on launching until the "
                         "clocks have settled, about 30 ms after an idle phase, and reports the count)")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--skip-decode", action="store_true")
    ap.add_argument("--skip-other-configs", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (reference dispatch for rocprofv3 --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no multi-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)

    from paper_2410_06577_amd import rodimus, workloads as wl
    rodimus.lib()                       # fail loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    w = wl.LAYER_1P6B
    scan, inp, o, S_T = bench_scan(w, args.steps, args.warmup, rodimus, wl, dev)
    out = {
        "metric": "chunk_scan_tokens_per_s", "value": scan["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": scan["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: chunk-scan forward B={w.B} T={w.T} H={w.H} dk={w.dk} dv={w.dv} "
                               f"chunk={w.chunk}, bf16 q/k/v/o, fp32 gates and state, S0 ~ N(0,0.1), S_T returned",
                   "global_batch": w.B, "seq_len": w.T, "parallelism": "single-gpu",
                   "kernel_path": {1: "generic", 2: "mfma"}.get(scan["path"], "none")},
        "roofline": {"bound": "hbm", "achieved": scan["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": scan["gbs"] / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES["scan_layer_1p6b"],
                     "traffic_source": "profiles/scan_mfma_kernel_layer_1p6b.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of the same "
                                       "launch, a counter figure from the profile run, not measured by this run)",
                     "kernel": "scan_mfma_kernel", "launch_ms": scan["launch_ms"], "algorithmic_bytes": scan["algo_bytes"],
                     "single_launch_ms": scan["single_launch_ms"], "settle_launches": scan["settle_launches"],
                     "settle_note": "untimed launches before the timed region: --warmup as given, continued until 150 ms of "
                                    "back-to-back launches have passed (GPU clocks ramp for ~30 ms after an idle phase)"},
        "mfma": {"achieved_causal": scan["tflops_causal"], "achieved_dense_tiles": scan["tflops_dense_tiles"],
                 "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": scan["tflops_causal"] / MFMA_BF16_PEAK_TFLOPS,
                 "note": "41.6 flop/B at dk=64: a single-pass scan is HBM-bound and cannot exceed ~13% of MFMA peak"},
    }
    if not args.skip_decode:
        dw = wl.DECODE
        dec = bench_decode(dw, rodimus, wl, dev)
        # same step over 512 sequences: 512 MiB of state, twice the last-level cache, i.e. every byte comes from HBM
        big = bench_decode(wl.DecodeWorkload("decode_512x16", N=512, H=dw.H, dk=dw.dk, dv=dw.dv, steps=200, ring=4, seed=5),
                           rodimus, wl, dev, warmup=50)
        out["decode"] = {
            "metric": "decode_step_GB_per_s", "value": dec["gbs"], "unit": "GB/s", "ms_per_step": dec["launch_ms"],
            "steps": dw.steps, "state_finite": dec["finite"],
            "workload": f"{dw.name}: {dw.N} sequences x H={dw.H} x ({dw.dk}x{dw.dv}) fp32 states, bf16 q/k/v/o, "
                        f"{dw.steps} chained steps",
            # the figure claimed against the HBM roofline is the all-HBM one: 512 sequences hold 512 MiB of state, twice the
            # last-level cache, so every byte of a step comes from and goes to HBM
            "roofline": {"bound": "hbm", "achieved": big["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": big["gbs"] / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES["decode_512x16"],
                         "traffic_source": "profiles/decode_step_kernel_256x16.md (counter figure of the profile run)",
                         "kernel": "decode_step_kernel (streaming variant)", "algorithmic_bytes": big["algo_bytes"],
                         "launch_ms": big["launch_ms"], "workload": "512 sequences x 16 heads, 200 chained steps"},
            "cache_assisted_256_sequences": {
                "GB_per_s_effective": dec["gbs"], "frac_of_hbm_peak": dec["gbs"] / HBM_PEAK_GBS, "ms_per_step": dec["launch_ms"],
                "algorithmic_bytes": dec["algo_bytes"], "traffic": MEASURED_TRAFFIC_BYTES["decode_256x16"],
                "traffic_source": "profiles/decode_step_kernel_256x16.md (counter figure of the profile run)",
                "note": "256 sequences hold exactly 256 MiB of state, the size of the last-level cache: chained steps find part "
                        "of it there (the same step with streaming accesses takes 96 us; the traffic counters sit in front of "
                        "that cache and read the full bytes), so this is a cache-assisted rate, not an HBM rate; with other "
                        "layers running between two steps of a model it would not be reached"},
        }
        if not args.skip_cpu_baseline:
            out["decode"]["cpu_baseline"] = decode_cpu_baseline(dw, wl)
    if not args.skip_other_configs:
        out["decode_small_batch"] = bench_decode_small(rodimus, wl, dev)
        out["ddts_gates"] = bench_gates(w, rodimus, wl, dev)
        out["short_conv"] = bench_short_conv(w, rodimus, wl, dev)
        del o, S_T
        zb, _, _, _ = bench_scan(w, args.steps, args.warmup, rodimus, wl, dev, zbeta=True)
        out["scan_fused_value_gate"] = {
            "entry_point": "rodimus_chunk_scan_fwd_zbeta", "workload": "layer_1p6b, value gate as bf16 pre-activation",
            "tokens_per_s": zb["tokens_per_s"], "ms_per_step": zb["launch_ms"], "algorithmic_bytes": zb["algo_bytes"],
            "GB_per_s": zb["gbs"], "hbm_frac": zb["gbs"] / HBM_PEAK_GBS}
        out["scan_fused_all_gates"] = bench_gated_scan(w, rodimus, wl, dev, args.steps, args.warmup)
        out["scan_block_output"] = bench_block_scan(w, rodimus, wl, dev, args.steps, args.warmup)
        out["scan_block_output"]["vs_plain_scan"] = out["scan_block_output"]["ms_per_step"] / scan["launch_ms"]
        probe = bench_stream_probe(rodimus, dev)
        out["hbm_stream_probe"] = probe
        out["roofline"]["vs_stream_probe"] = scan["gbs"] / probe["four_reads_per_write"]["GB_per_s"]
        if "decode" in out:
            out["decode"]["roofline"]["vs_stream_probe"] = out["decode"]["roofline"]["achieved"] / probe["one_read_per_write"]["GB_per_s"]
        out["scan_whole_block"] = bench_whole_block_scan(w, rodimus, wl, dev, args.steps, args.warmup)
        out["scan_whole_block"]["vs_plain_scan"] = out["scan_whole_block"]["ms_per_step"] / scan["launch_ms"]
        out["scan_backward"] = bench_backward(w, rodimus, wl, dev, args.steps, args.warmup)
        zb_bwd = bench_backward(w, rodimus, wl, dev, args.steps, args.warmup, zbeta=True)
        out["scan_backward_fused_value_gate"] = {k: zb_bwd[k] for k in ("entry_point", "ms_per_step", "tokens_per_s", "algorithmic_bytes",
                                                                       "GB_per_s", "hbm_frac", "finite")}
        out["scan_backward_all_gates"] = bench_backward_gated(w, rodimus, wl, dev, args.steps, args.warmup)
        # the same layer at a micro-batch of two sequences: too few (batch, head) pairs to fill the chip, the call is cut
        # along the sequence
        import dataclasses
        small = dataclasses.replace(w, name="layer_1p6b_micro_batch_2", B=2)
        mb = bench_backward(small, rodimus, wl, dev, args.steps, args.warmup)
        out["scan_backward_micro_batch"] = {"workload": f"B={small.B} T={small.T} H={small.H} dk={small.dk} dv={small.dv}",
                                            **{k: mb[k] for k in ("ms_per_step", "tokens_per_s", "GB_per_s", "hbm_frac", "finite")}}
        out["scan_backward_few_long_sequences"] = bench_backward_few_long(w, rodimus, wl, dev, args.steps, args.warmup)
        out["serving_prefill_varlen"] = bench_varlen(w, rodimus, wl, dev, args.steps, args.warmup)
        lf = bench_varlen(w, rodimus, wl, dev, args.steps, args.warmup, longest_first=True)
        out["serving_prefill_varlen"]["sequences_sorted_longest_first"] = {
            k: lf[k] for k in ("ms_per_step", "tokens_per_s", "GB_per_s", "hbm_frac")}
        out["serving_prefill_whole_block"] = bench_varlen_whole_block(w, rodimus, wl, dev, args.steps, args.warmup)
        # few long sequences: the packed call lasts as long as its longest sequence unless the kernels cut the sequences
        few = bench_varlen(w, rodimus, wl, dev, args.steps, args.warmup, n_seq=8)
        few_cut = bench_varlen(w, rodimus, wl, dev, args.steps, args.warmup, n_seq=8, cut=True)
        out["serving_prefill_few_long_sequences"] = {**few_cut, "uncut_ms_per_step": few["ms_per_step"]}
        others = {}
        for ow in (wl.MID, wl.LONG_CONTEXT):
            r, _, _, _ = bench_scan(ow, args.steps, args.warmup, rodimus, wl, dev)
            others[ow.name] = {"workload": f"B={ow.B} T={ow.T} H={ow.H} dk={ow.dk} dv={ow.dv} chunk={ow.chunk}",
                               "tokens_per_s": r["tokens_per_s"], "ms_per_step": r["launch_ms"], "GB_per_s": r["gbs"],
                               "hbm_frac": r["gbs"] / HBM_PEAK_GBS, "kernel_path": {1: "generic", 2: "mfma"}.get(r["path"])}
        out["other_scan_configs"] = others
        scan2, inp, o, S_T = None, inp, *bench_scan_outputs(w, inp, rodimus, dev)
    if not args.skip_cpu_baseline:
        base, parity = cpu_baseline(w, inp, o, S_T)
        out["cpu_baseline"] = base
        out["parity_vs_oracle"] = parity
    print(json.dumps(out))


if __name__ == "__main__":
    main()
