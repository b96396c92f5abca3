#!/usr/bin/env python3
"""Benchmark of the SERQ linear hot path on one MI355X.

A step is one pass of the whole online path over one batch of synthetic
activations that are already resident in HBM: serq_quantize_act (flatten +
per-token INT8 quantisation) followed by serq_linear (INT4-weight int8-MFMA
GEMM with the rank-128 compensation and the dequantising epilogue fused).
Workload: the up projection of the MLP pair, W4A8, M = 4096 tokens,
K = 4096 -> N = 11008, r = 128, bf16 in / bf16 out.

Before anything is timed the step runs untimed for 0.15 s: coming out of idle the
part takes about 40 ms of load to reach its sustained clocks, and a 50-step run
would otherwise sit entirely inside that ramp.

Prints ONE JSON line.  `value` is 2*M*N*K / step time in TOPS.  `roofline`
prices the dominant kernel (serq_linear) against the int8 MFMA peak using its
own launch durations, measured with HIP events on the launch stream inside the
timed region.  `measured_peaks` says what the part sustains with nothing in the way (an MFMA-only
loop on this layer's operand bytes; read-only kernels), and the fractions of those
are reported next to the fractions of the datasheet peaks.
`decode` reports the M = 1 weight-streaming kernel in GB/s with
the weight copies rotated so that the working set exceeds the Infinity Cache;
the launches are replayed from a HIP graph, as a serving loop would issue them.
`cpu_baseline` is the NumPy oracle timed on whole passes (about 10 s) over the same
workload on this host's cores.

`--sweep` times every benchmark configuration instead (one JSON line per row).
`--calibrate-copy` runs nothing but a plain device copy of a known size; it
exists so that the FETCH_SIZE / WRITE_SIZE counters of a profiler run of this
script can be scaled to bytes.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads  # noqa: E402
from paper_2603_08185_amd import binding as serq  # noqa: E402

FP4_PEAK_TFLOPS = 10100.0  # dense FP4 MFMA, MI355X datasheet
INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA, 5.0 POP/s
HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, 8 TB/s

# HBM traffic of one serq_linear launch of the benchmark workload, from two counter runs
# (FETCH_SIZE, then WRITE_SIZE) of this script scaled by the same counters of --calibrate-copy;
# the runs and the arithmetic are in profiles/serq_mfma_kernel_cfg3_up_M4096_hbm_traffic.md.
# 103 150 FETCH_SIZE counts x 2048 B + 88 088 WRITE_SIZE counts x 1024 B.
LINEAR_TRAFFIC_BYTES = 103150 * 2048 + 88088 * 1024
# the same two counters for serq_mx_kernel on the MXFP4 up projection: 78 736 and 88 098 counts
MX_TRAFFIC_BYTES = 78736 * 2048 + 88098 * 1024


def _events(n):
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def spin_up(fn, seconds: float = 0.15):
    """Untimed load before any measurement: after idling, the part needs about 40 ms of work to reach its
    sustained clocks (the first 20 ms of this benchmark's step run 25 % slower than the steady state)."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(20):
            fn()
        torch.cuda.synchronize()


def bench_prefill(steps: int, warmup: int):
    spec = workloads.config3("up", 4096)
    L = workloads.make_layer(spec)
    dev = "cuda:0"
    pk = serq.pack_weights(L["W"].to(dev), L["s"].to(dev), spec.r, r_dtype=torch.bfloat16, want_R=False, want_Rp=False)
    Rp = serq.pack_lowrank(L["R"].to(dev))
    Xhat = workloads.permute_channels(L["X"], pk.perm.cpu().numpy()).to(dev)
    M, N, K = spec.M, spec.N, spec.K
    Xq = torch.empty(M * K, dtype=torch.uint8, device=dev)
    scale = torch.empty(M, dtype=torch.float32, device=dev)
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)

    def step():
        serq.quantize_act(Xhat, pk.s_inv, spec.abits, Xq=Xq, scale=scale)
        serq.linear(Xq, scale, spec.abits, pk.Wq, pk.wscale, M, N, K, Rp=Rp, r=spec.r, Y=Y)

    spin_up(step)
    for _ in range(warmup):
        step()
    ev = _events(2 * steps + 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        serq.quantize_act(Xhat, pk.s_inv, spec.abits, Xq=Xq, scale=scale)
        ev[2 * i + 1].record()
        serq.linear(Xq, scale, spec.abits, pk.Wq, pk.wscale, M, N, K, Rp=Rp, r=spec.r, Y=Y)
        ev[2 * i + 2].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    total_ms = ev[0].elapsed_time(ev[-1])
    q_ms = float(np.mean([ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(steps)]))
    l_ms = float(np.mean([ev[2 * i + 1].elapsed_time(ev[2 * i + 2]) for i in range(steps)]))
    ops = 2.0 * M * N * K
    qbytes = 2.0 * M * K + M * K * spec.abits / 8 + 4 * M
    return {
        "spec": spec, "ms_per_step": total_ms / steps, "wall_ms_per_step": wall * 1e3 / steps,
        "quant_ms": q_ms, "linear_ms": l_ms, "ops": ops,
        "tops_step": ops / (total_ms / steps * 1e-3) / 1e12,
        "tops_linear": ops / (l_ms * 1e-3) / 1e12,
        "quant_gbs": qbytes / (q_ms * 1e-3) / 1e9,
        "layer": (L, pk), "Xq": Xq,
    }


def bench_mx(steps: int, warmup: int, which: str = "up"):
    """The MXFP4 variant of the layer on the headline shape: one JSON line of its own (`--mx`)."""
    spec = workloads.config3(which, 4096)
    L = workloads.make_layer(spec, want=("X", "s", "W"))
    dev = "cuda:0"
    pk = serq.mx_pack_weights(L["W"].to(dev), L["s"].to(dev), spec.r)
    Xhat = workloads.permute_channels(L["X"], pk.perm.cpu().numpy()).to(dev)
    M, N, K, r = spec.M, spec.N, spec.K, spec.r
    Xq = torch.empty(M * K // 2, dtype=torch.uint8, device=dev)
    xsc = torch.empty(serq.lib().serq_mx_act_scale_bytes(M, K), dtype=torch.uint8, device=dev)
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)

    def quant():
        serq.mx_quantize_act(Xhat, pk.s_inv, Xq=Xq, xsc=xsc)

    def lin():
        serq.mx_linear(Xq, xsc, pk.Wq, pk.wsc, M, N, K, Rq=pk.Rq, rsc=pk.rsc, r=r, Y=Y)

    def step():
        quant()
        lin()

    spin_up(step)
    for _ in range(warmup):
        step()
    ev = _events(2 * steps + 1)
    torch.cuda.synchronize()
    ev[0].record()
    for i in range(steps):
        quant()
        ev[2 * i + 1].record()
        lin()
        ev[2 * i + 2].record()
    torch.cuda.synchronize()
    total_ms = ev[0].elapsed_time(ev[-1])
    q_ms = float(np.mean([ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(steps)]))
    l_ms = float(np.mean([ev[2 * i + 1].elapsed_time(ev[2 * i + 2]) for i in range(steps)]))
    ops = 2.0 * M * N * K
    qbytes = 2.0 * M * K + M * K / 2 + M * K / 32
    tf_lin = ops / (l_ms * 1e-3) / 1e12
    # the decode-sized call (M = 1) on the same weights, rotated over > 640 MB of copies, replayed from a graph
    per_copy = pk.Wq.numel() + pk.wsc.numel()
    ncopy = int(np.ceil(640e6 / per_copy))
    copies = [(pk.Wq, pk.wsc, pk.Rq, pk.rsc)] + [(pk.Wq.clone(), pk.wsc.clone(), pk.Rq.clone(), pk.rsc.clone())
                                                 for _ in range(ncopy - 1)]
    Xq1, xsc1 = serq.mx_quantize_act(Xhat[:1].contiguous(), pk.s_inv)
    Y1 = torch.empty((1, N), dtype=torch.bfloat16, device=dev)
    ws1 = serq.mx_workspace(1, N, K, dev)

    def dec(i):
        wq, wsc_, rq, rsc_ = copies[i % ncopy]
        serq.mx_linear(Xq1, xsc1, wq, wsc_, 1, N, K, Rq=rq, rsc=rsc_, r=r, Y=Y1, ws=ws1)

    dec(0)
    spin_up(lambda: dec(0), 0.05)
    d_us = min(_time_launches(dec, 4 * ncopy, graph=True) for _ in range(3))
    d_bytes = N * K / 2 + N * K / 32 + N * 64 * ((r + 63) // 64) * (0.5 + 1 / 32) + K / 2 + K / 32 + 2.0 * N
    del copies
    # what the part sustains on nothing but FP4 MFMAs fed with this layer's own code bytes
    ops_buf = torch.cat([pk.Wq[:16384].reshape(256, 4, 16), Xq[:16384].reshape(256, 4, 16)], dim=1).contiguous()
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    iters, wgs = 2000, 1024
    run = lambda: serq.bench_mfma_fp4_peak(ops_buf, iters, wgs, sink)
    spin_up(run, 0.1)
    fp4_tf = 2.0 * 32 * 32 * 64 * 16 * iters * 4 * wgs / _time_launches(lambda i: run(), 5) / 1e6
    return {
        "variant": "mxfp4", "metric": "fused SERQ linear in MXFP4, TFLOP/s (M=4096), 1 MI355X",
        "value": round(ops / (total_ms / steps * 1e-3) / 1e12, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": round(total_ms / steps, 5), "higher_is_better": True,
        "dtype": "fp4 (E2M1 x E8M0 block scales), fp32 accumulation", "data": "synthetic",
        "config": {"workload": f"configs[2]: MLP {which} projection in MXFP4 (weights, activations, compensation "
                               "matrix), M=4096, bf16 in/out; step = serq_mx_quantize_act + serq_mx_linear",
                   "M": M, "K": K, "N": N, "r": r},
        "roofline": {"bound": "mfma", "kernel": "serq_mx_kernel (serq_mx_linear)", "achieved": round(tf_lin, 2),
                     "peak": FP4_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(tf_lin / FP4_PEAK_TFLOPS, 4),
                     "traffic": MX_TRAFFIC_BYTES if which == "up" else None, "kernel_ms": round(l_ms, 5),
                     "frac_of_measured_mfma_peak": round(tf_lin / fp4_tf, 4)},
        "measured_peaks": {"mfma_fp4_tflops": round(fp4_tf, 1), "mfma_operands": "this layer's codes"},
        "quantize_act": {"ms": round(q_ms, 5), "gbs": round(qbytes / (q_ms * 1e-3) / 1e9, 1),
                         "frac_hbm_peak": round(qbytes / (q_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "decode": {"workload": f"the same layer, M=1 (serq_skinny_mx_kernel), {ncopy} weight copies", "bytes": int(d_bytes),
                   "us_hbm": round(d_us, 3), "gbs_hbm": round(d_bytes / d_us / 1e3, 1),
                   "frac_hbm_peak": round(d_bytes / d_us / 1e3 / HBM_PEAK_GBS, 4)},
    }


def decode_bytes(spec) -> float:
    """Algorithmic HBM bytes of one decode-sized serq_linear call."""
    M, N, K, r = spec.M, spec.N, spec.K, spec.r
    out_b = 2 if spec.out_dtype != "fp32" else 4
    return N * K / 2 + 2.0 * r * N + 4 * N + M * K * spec.abits / 8 + 4 * M + M * N * out_b


def read_stick(nbytes: int) -> float:
    """GB/s of a launch that only reads `nbytes` (rotating over > 640 MB of distinct buffers, replayed from a graph):
    what a decode-sized call of that many bytes could reach at best on this part."""
    dev = "cuda:0"
    nbytes = nbytes // 16 * 16
    ncopy = int(np.ceil(640e6 / nbytes))
    big = torch.empty(ncopy * nbytes, dtype=torch.uint8, device=dev).fill_(1)
    views = [big[i * nbytes:(i + 1) * nbytes] for i in range(ncopy)]
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    rd = lambda i: serq.bench_read(views[i % ncopy], nbytes, 2048, sink)
    spin_up(lambda: rd(0), 0.05)
    us = _time_launches(rd, max(4 * ncopy, 20), graph=True)
    return nbytes / us / 1e3


def bench_decode(L, pk, reps: int = 5, spec=None):
    """M = 1 on the given layer (default: the benchmark's own); weights + R rotated over > 640 MB of distinct copies."""
    dev = "cuda:0"
    spec = spec or workloads.config3("up", 1)
    M, N, K = 1, spec.N, spec.K
    X1 = workloads.make_layer(spec, want=("X",))["X"]
    Xhat = workloads.permute_channels(X1, pk.perm.cpu().numpy()).to(dev)
    Xq, scale = serq.quantize_act(Xhat, pk.s_inv, spec.abits)
    Rp0 = serq.pack_lowrank(L["R"].to(dev))
    per_copy = pk.Wq.numel() + Rp0.numel()
    ncopy = int(np.ceil(640e6 / per_copy))
    Wqs = [pk.Wq.clone() for _ in range(ncopy)]
    Rps = [Rp0.clone() for _ in range(ncopy)]
    ws = serq.workspace(M, N, K, spec.r, spec.abits, dev)
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    n = 4 * ncopy

    def launches(rotate: bool):
        for i in range(n):
            j = i % ncopy if rotate else 0
            serq.linear(Xq, scale, spec.abits, Wqs[j], pk.wscale, M, N, K, Rp=Rps[j], r=spec.r, Y=Y, ws=ws)

    def timed(fn):
        e0, e1 = _events(2)
        torch.cuda.synchronize()
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    spin_up(lambda: launches(True), 0.05)
    side = torch.cuda.Stream()          # graph capture needs a non-default stream (default priority)
    graphs = {}
    for rotate in (True, False):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                launches(rotate)
        graphs[rotate] = g
    torch.cuda.synchronize()
    spin_up(graphs[True].replay, 0.05)
    for g in graphs.values():
        g.replay()
    cold = min(timed(graphs[True].replay) for _ in range(reps))
    warm = min(timed(graphs[False].replay) for _ in range(reps))
    cold_stream = min(timed(lambda: launches(True)) for _ in range(reps))
    b = decode_bytes(spec)
    return {"workload": spec.name, "bytes": b, "copies": ncopy,
            "us_hbm": cold * 1e3, "gbs_hbm": b / (cold * 1e-3) / 1e9,
            "us_cache_warm": warm * 1e3, "gbs_cache_warm": b / (warm * 1e-3) / 1e9,
            "us_hbm_stream_launch": cold_stream * 1e3,
            "frac_hbm_peak": b / (cold * 1e-3) / 1e9 / HBM_PEAK_GBS}


def measured_peaks(pk, Xq, spec):
    """What this part sustains with nothing in the way: an MFMA-only loop fed with this layer's own operand
    bytes (weight codes widened to 16q as the kernel feeds them, token codes as they are), and read-only kernels
    of the decode call's size (rotating over > 640 MB, replayed from a graph) and of 1 GiB."""
    dev = "cuda:0"
    w = serq.unpack_weights(pk.Wq, spec.N, spec.K)[:256, :64].to(torch.int16) * 16
    x = serq.unpack_act(Xq, spec.abits, spec.M, spec.K)[:256, :64]
    ops_buf = torch.cat([w.to(torch.int8).reshape(256, 4, 16), x.reshape(256, 4, 16)], dim=1).contiguous()
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    iters, wgs = 2000, 1024
    run = lambda: serq.bench_mfma_peak(ops_buf, iters, wgs, sink)
    spin_up(run, 0.1)
    t_us = _time_launches(lambda i: run(), 5)
    mfma_tops = 2.0 * 32 ** 3 * 16 * iters * 4 * wgs / t_us / 1e6
    nbytes = int(decode_bytes(workloads.config3("up", 1))) // 16 * 16
    ncopy = int(np.ceil(640e6 / nbytes))
    big = torch.empty(max(ncopy * nbytes, 1 << 30), dtype=torch.uint8, device=dev).fill_(1)
    views = [big[i * nbytes:(i + 1) * nbytes] for i in range(ncopy)]
    rd = lambda i: serq.bench_read(views[i % ncopy], nbytes, 2048, sink)
    spin_up(lambda: rd(0), 0.05)
    small_us = _time_launches(rd, 4 * ncopy, graph=True)
    large_us = _time_launches(lambda i: serq.bench_read(big, 1 << 30, 16384, sink), 3)
    return {"mfma_int8_tops": round(mfma_tops, 1), "mfma_operands": "this layer's codes (weights x16, tokens)",
            "read_gbs_decode_size": round(nbytes / small_us / 1e3, 1), "read_bytes_decode_size": nbytes,
            "read_gbs_1GiB": round((1 << 30) / large_us / 1e3, 1)}


def cpu_baseline(L, n_tokens: int = 4096, min_seconds: float = 10.0):
    """The oracle, as it stands, on the workload's tokens (all N, all K): whole passes until min_seconds have gone by."""
    from threadpoolctl import threadpool_info
    from oracle import serq_oracle as orc
    spec = workloads.config3("up", 4096)
    W = L["W"].float().numpy()
    pk = orc.pack_weights(W, L["s"].numpy(), spec.r)           # offline: not timed
    R = L["R"].double().numpy()
    X = L["X"][:n_tokens].float().numpy()[:, pk["perm"]]
    passes = 0
    t0 = time.perf_counter()
    while True:
        Xq, scale = orc.quantize_act(X, pk["s_inv"], spec.abits)
        Y = orc.linear(Xq, scale, pk["Wq"], pk["wscale"], R)
        passes += 1
        dt = time.perf_counter() - t0
        if dt >= min_seconds or passes >= 64:
            break
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    ops = 2.0 * n_tokens * spec.N * spec.K * passes
    return {"value": ops / dt / 1e12, "unit": "TOPS", "cores": int(threads), "kind": "oracle",
            "sample": f"{passes} passes over {n_tokens} of 4096 tokens, full N=11008, K=4096, r=128 "
                      f"(quantize_act + gemm + epilogue), {dt:.1f} s", "host_cpus": len(os.sched_getaffinity(0))}, Y


def _time_launches(fn, n: int, reps: int = 3, graph: bool = False) -> float:
    """Best-of-reps average time of n back-to-back launches of fn(i), in microseconds.  With graph=True the
    n launches are captured once and replayed (short kernels: the Python call costs more than the launch)."""
    run = lambda: [fn(i) for i in range(n)]
    if graph:
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                run()
        torch.cuda.synchronize()
        g.replay()
        run = g.replay
    best = float("inf")
    for _ in range(reps):
        e0, e1 = _events(2)
        torch.cuda.synchronize()
        e0.record()
        run()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) * 1e3 / n)
    return best


def sweep(only: str = ""):
    """Every benchmark configuration, one JSON line each: quantize_act and serq_linear timed separately
    (HIP events around back-to-back launches; decode-sized shapes rotate over copies of the weights that
    together exceed the Infinity Cache and are replayed from a HIP graph), with the roofline that bounds the row."""
    dev = "cuda:0"
    rows = [workloads.config2()]
    rows += [workloads.config3(w, M) for w in ("up", "down") for M in (1, 16, 256, 4096)]
    rows += [workloads.config4(M) for M in (1, 4, 32)]
    rows += [workloads.config5(layer, r) for layer in workloads.config5_layers() for r in (0, 32, 64, 128, 256)]
    if only:
        rows = [r_ for r_ in rows if any(tok in r_.name for tok in only.split(","))]
    cache = {}
    for spec in rows:
        key = (spec.cfg, spec.N, spec.K, spec.abits, spec.seed_index)
        if key not in cache:                        # weights depend on the layer, not on M or r
            cache.clear()
            L = workloads.make_layer(spec, want=("s", "W"))
            cache[key] = serq.pack_weights(L["W"].to(dev), L["s"].to(dev), 0, want_R=False, want_Rp=False)
        pk = cache[key]
        M, N, K, r = spec.M, spec.N, spec.K, spec.r
        X = workloads.make_layer(spec, want=("X",))["X"]
        Xhat = workloads.permute_channels(X, pk.perm.cpu().numpy()).to(dev)
        Rp = Rq = None
        if r:
            g = torch.Generator().manual_seed(1000 * spec.cfg + 7)
            Rh = (torch.randn((r, N), generator=g) * 0.01).to(torch.bfloat16).to(dev)
            Rp = serq.pack_lowrank(Rh)
            Rq = serq.pack_lowrank_q4(Rh)                 # the same matrix on the 4-bit grid (Eq. 7, second line)
        Xq = torch.empty(M * K * spec.abits // 8, dtype=torch.uint8, device=dev)
        scale = torch.empty(M, dtype=torch.float32, device=dev)
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        ws = serq.workspace(M, N, K, r, spec.abits, dev)
        small = M <= 32
        ncopy = 1
        if small:
            per_copy = pk.Wq.numel() + (Rp.numel() if Rp is not None else 0)
            ncopy = int(np.ceil(640e6 / per_copy))
        Wqs = [pk.Wq] + [pk.Wq.clone() for _ in range(ncopy - 1)]
        Rps = [Rp] + [Rp.clone() if Rp is not None else None for _ in range(ncopy - 1)]
        Rqs = [Rq] + [Rq.clone() if Rq is not None else None for _ in range(ncopy - 1)]
        n = max(20, 2 * ncopy)

        def q(i):
            serq.quantize_act(Xhat, pk.s_inv, spec.abits, Xq=Xq, scale=scale)

        def lin(i):
            j = i % ncopy
            serq.linear(Xq, scale, spec.abits, Wqs[j], pk.wscale, M, N, K, Rp=Rps[j], r=r, Y=Y, ws=ws)

        def lin_q4r(i):
            j = i % ncopy
            serq.linear(Xq, scale, spec.abits, Wqs[j], pk.wscale, M, N, K, Rp=Rqs[j], r=r, r_dtype=serq.I4, Y=Y, ws=ws)

        spin_up(lambda: lin(0), 0.05)
        q(0)
        q_us = _time_launches(q, n, graph=small)
        l_us = _time_launches(lin, n, graph=small)
        row = {"workload": spec.name, "abits": spec.abits, "M": M, "K": K, "N": N, "r": r,
               "quantize_act_us": round(q_us, 2), "serq_linear_us": round(l_us, 2), "layer_us": round(q_us + l_us, 2)}
        if r:
            lin_q4r(0)
            row["serq_linear_q4r_us"] = round(_time_launches(lin_q4r, n, graph=small), 2)
        if "down" in spec.name:
            # the down projection's input quantised where it is made: silu(gate) * up -> codes in one pass
            gg = torch.Generator().manual_seed(1000 * spec.cfg + 11)
            G = (torch.randn((M, K), generator=gg) * 2.5).to(torch.bfloat16).to(dev)
            U = (torch.randn((M, K), generator=gg) * 1.5).to(torch.bfloat16).to(dev)

            def sq(i):
                serq.swiglu_quantize_act(G, U, pk.s_inv, spec.abits, Xq=Xq, scale=scale)

            sq(0)
            sq_us = _time_launches(sq, n, graph=small)
            sq_bytes = 4.0 * M * K + M * K * spec.abits / 8 + 4 * M
            row["swiglu_quantize_act"] = {"us": round(sq_us, 2), "gbs": round(sq_bytes / sq_us / 1e3, 1),
                                          "frac_hbm_peak": round(sq_bytes / sq_us / 1e3 / HBM_PEAK_GBS, 4)}
            if not small:
                xsc_g = torch.empty(max(serq.lib().serq_mx_act_scale_bytes(M, K), 16), dtype=torch.uint8, device=dev)
                Xq4_g = torch.empty(M * K // 2, dtype=torch.uint8, device=dev)

                def msq(i):
                    serq.mx_swiglu_quantize_act(G, U, pk.s_inv, Xq=Xq4_g, xsc=xsc_g)

                msq(0)
                msq_us = _time_launches(msq, n)
                msq_bytes = 4.0 * M * K + M * K / 2 + M * K / 32
                row["mx_swiglu_quantize_act"] = {"us": round(msq_us, 2), "gbs": round(msq_bytes / msq_us / 1e3, 1),
                                                 "frac_hbm_peak": round(msq_bytes / msq_us / 1e3 / HBM_PEAK_GBS, 4)}
                del xsc_g, Xq4_g
            del G, U
        if small:
            b = decode_bytes(spec)
            row.update({"bound": "hbm", "gbs": round(b / l_us / 1e3, 1), "frac": round(b / l_us / 1e3 / HBM_PEAK_GBS, 4)})
            # the same call in MXFP4 (weight-streaming kernel on the FP4 units), weights rotated the same way
            rm = 32 * (r // 32)
            Lw = workloads.make_layer(spec, want=("s", "W"))
            mpk = serq.mx_pack_weights(Lw["W"].to(dev), Lw["s"].to(dev), rm, perm_in=pk.perm)
            del Lw
            per_copy = mpk.Wq.numel() + mpk.wsc.numel()
            mcopy = int(np.ceil(640e6 / per_copy))
            mW = [(mpk.Wq, mpk.wsc, mpk.Rq, mpk.rsc)] + [
                (mpk.Wq.clone(), mpk.wsc.clone(), None if mpk.Rq is None else mpk.Rq.clone(),
                 None if mpk.rsc is None else mpk.rsc.clone()) for _ in range(mcopy - 1)]
            Xq4, xsc = serq.mx_quantize_act(Xhat, mpk.s_inv)
            mws = serq.mx_workspace(M, N, K, dev)

            def mlin_d(i):
                wq, wsc_, rq, rsc_ = mW[i % mcopy]
                serq.mx_linear(Xq4, xsc, wq, wsc_, M, N, K, Rq=rq, rsc=rsc_, r=rm, Y=Y, ws=mws)

            mlin_d(0)
            md_us = _time_launches(mlin_d, max(20, 2 * mcopy), graph=True)
            mb = N * K / 2 + N * K / 32 + (N * 64 * ((rm + 63) // 64) * (0.5 + 1 / 32) if rm else 0) + M * K / 2 + M * K / 32 + 2.0 * M * N
            row["mxfp4"] = {"r": rm, "serq_mx_linear_us": round(md_us, 2), "bytes": int(mb), "gbs": round(mb / md_us / 1e3, 1),
                            "frac_hbm_peak": round(mb / md_us / 1e3 / HBM_PEAK_GBS, 4)}
            del mW, mpk
        else:
            ops = 2.0 * M * N * K
            row.update({"bound": "mfma", "tops": round(ops / l_us / 1e6, 1),
                        "frac": round(ops / l_us / 1e6 / INT8_PEAK_TOPS, 4)})
            # the same layer in MXFP4 (weights, activations and compensation matrix), on the FP4 units
            rm = 32 * (r // 32)
            Lw = workloads.make_layer(spec, want=("s", "W"))
            mpk = serq.mx_pack_weights(Lw["W"].to(dev), Lw["s"].to(dev), rm, perm_in=pk.perm)
            del Lw
            xsc = torch.empty(max(serq.lib().serq_mx_act_scale_bytes(M, K), 16), dtype=torch.uint8, device=dev)
            Xq4 = torch.empty(M * K // 2, dtype=torch.uint8, device=dev)

            def mq(i):
                serq.mx_quantize_act(Xhat, mpk.s_inv, Xq=Xq4, xsc=xsc)

            mws2 = serq.mx_workspace(M, N, K, dev)                # K slices for few tokens and a long K

            def mlin(i):
                serq.mx_linear(Xq4, xsc, mpk.Wq, mpk.wsc, M, N, K, Rq=mpk.Rq, rsc=mpk.rsc, r=rm, Y=Y, ws=mws2)

            mq(0)
            spin_up(lambda: mlin(0), 0.05)
            mq_us = _time_launches(mq, n)
            ml_us = _time_launches(mlin, n)
            row["mxfp4"] = {"r": rm, "quantize_act_us": round(mq_us, 2), "serq_mx_linear_us": round(ml_us, 2),
                            "tflops": round(ops / ml_us / 1e6, 1), "frac_of_fp4_peak": round(ops / ml_us / 1e6 / FP4_PEAK_TFLOPS, 4)}
            del mpk
        if K % 128 == 0:
            # the accuracy-table setting: group-128 weight scales + asymmetric activations (serq_g128_linear)
            Lw = workloads.make_layer(spec, want=("s", "W"))
            gpk = serq.g128_pack_weights(Lw["W"].to(dev), Lw["s"].to(dev), 0, perm_in=pk.perm)
            del Lw
            gcopy = int(np.ceil(640e6 / (gpk.Wq.numel() + gpk.gscale.numel()))) if small else 1
            gW = [(gpk.Wq, gpk.gscale)] + [(gpk.Wq.clone(), gpk.gscale.clone()) for _ in range(gcopy - 1)]
            za = torch.empty(M, dtype=torch.int32, device=dev)

            def gq(i):
                serq.quantize_act_asym(Xhat, gpk.s_inv, spec.abits, Xq=Xq, scale=scale, zero=za)

            def glin(i):
                wq, gs_ = gW[i % gcopy]
                serq.g128_linear(Xq, scale, za, spec.abits, wq, gs_, gpk.wsum, M, N, K, Rp=Rps[0], r=r, Y=Y)

            gq(0)
            glin(0)
            gq_us = _time_launches(gq, n, graph=small)
            gl_us = _time_launches(glin, max(n, 2 * gcopy), graph=small)
            g = {"quantize_act_asym_us": round(gq_us, 2), "serq_g128_linear_us": round(gl_us, 2)}
            if small:
                gb = decode_bytes(spec) + N * (K // 128) * 2 + 4 * N
                g.update({"bytes": int(gb), "gbs": round(gb / gl_us / 1e3, 1), "frac_hbm_peak": round(gb / gl_us / 1e3 / HBM_PEAK_GBS, 4)})
            else:
                g.update({"tops": round(2.0 * M * N * K / gl_us / 1e6, 1),
                          "frac_of_int8_peak": round(2.0 * M * N * K / gl_us / 1e6 / INT8_PEAK_TOPS, 4)})
            row["g128_asym"] = g
            del gW, gpk
        if spec.cfg == 5 and r == 0 and spec.abits == 4 and ("_o_" in spec.name or "_down_" in spec.name):
            # experiment: the same INT32 sums from one plain tiled kernel by two operand routes -- 4-bit codes
            # widened for the int8 instruction, and FP6 (E2M3) codes on the block-scaled instruction
            codes_w = serq.unpack_weights(pk.Wq, N, K)
            codes_x = serq.unpack_act(Xq, 4, M, K)
            W6 = serq.fp6_pack_weights(codes_w)
            X6 = serq.fp6_pack_act(codes_x)
            del codes_w, codes_x
            acc = torch.empty((M, N), dtype=torch.int32, device=dev)
            serq.proto_gemm_i32(Xq, pk.Wq, False, M, N, K, acc=acc)
            spin_up(lambda: serq.proto_gemm_i32(X6, W6, True, M, N, K, acc=acc), 0.05)
            i8_us = _time_launches(lambda i: serq.proto_gemm_i32(Xq, pk.Wq, False, M, N, K, acc=acc), n)
            f6_us = _time_launches(lambda i: serq.proto_gemm_i32(X6, W6, True, M, N, K, acc=acc), n)
            i8b_us = _time_launches(lambda i: serq.proto_gemm_i32(Xq, pk.Wq, False, M, N, K, acc=acc), n)
            row["fp6_experiment"] = {"kernel": "proto_gemm_kernel (plain 128x128 tiles, INT32 out)",
                                     "int8_route_us": round(min(i8_us, i8b_us), 2), "fp6_route_us": round(f6_us, 2),
                                     "int8_route_tops": round(2.0 * M * N * K / min(i8_us, i8b_us) / 1e6, 1),
                                     "fp6_route_tops": round(2.0 * M * N * K / f6_us / 1e6, 1)}
            del W6, X6, acc
        print(json.dumps(row), flush=True)
        del Wqs, Rps, Rqs


def calibrate_copy(nbytes: int = 1 << 30, reps: int = 3):
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0").fill_(1)
    dst = torch.empty_like(src)
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"calibrate_copy_bytes": nbytes, "launches": reps}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-decode", action="store_true", help="skip the M=1 decode leg")
    ap.add_argument("--calibrate-copy", action="store_true", help="only run a plain 1 GiB device copy (counter calibration)")
    ap.add_argument("--no-mx", action="store_true", help="skip the MXFP4 leg of the default run")
    ap.add_argument("--mx", nargs="?", const="up", default=None, choices=["up", "down"],
                    help="time the MXFP4 variant of the layer on the headline shape (up, default) or its down projection instead")
    ap.add_argument("--only", default="", help="with --sweep: comma-separated substrings of the workload names to time")
    ap.add_argument("--sweep", action="store_true", help="time every benchmark configuration (one JSON line per row) instead of the headline step")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    serq.lib()
    if a.calibrate_copy:
        calibrate_copy()
        return
    if a.sweep:
        sweep(a.only)
        return
    if a.mx:
        print(json.dumps(bench_mx(a.steps, a.warmup, a.mx)))
        return

    pre = bench_prefill(a.steps, a.warmup)
    spec = pre["spec"]
    L, pk = pre["layer"]
    out = {
        "metric": "fused SERQ linear TOPS (M=4096, 4096x11008) + decode GB/s (M=1), 1 MI355X",
        "value": round(pre["tops_step"], 2), "unit": "TOPS",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(pre["ms_per_step"], 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "configs[2]: MLP up projection W4A8, M=4096, K=4096->N=11008, r=128, bf16 in/out; "
                               "step = serq_quantize_act + serq_linear",
                   "M": spec.M, "K": spec.K, "N": spec.N, "r": spec.r, "abits": spec.abits},
        "roofline": {"bound": "mfma", "kernel": "serq_mfma_kernel<8, 2> (serq_linear; W4A8, bf16 R)",
                     "achieved": round(pre["tops_linear"], 2), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                     "frac": round(pre["tops_linear"] / INT8_PEAK_TOPS, 4), "traffic": LINEAR_TRAFFIC_BYTES,
                     "traffic_source": "constant from profiles/serq_mfma_kernel_cfg3_up_M4096_hbm_traffic.md (two "
                                       "rocprofv3 --pmc runs of this command, FETCH_SIZE then WRITE_SIZE, scaled by "
                                       "--calibrate-copy); not measured in this run",
                     "kernel_ms": round(pre["linear_ms"], 5)},
        "quantize_act": {"ms": round(pre["quant_ms"], 5), "gbs": round(pre["quant_gbs"], 1),
                         "frac_hbm_peak": round(pre["quant_gbs"] / HBM_PEAK_GBS, 4)},
    }
    mp = measured_peaks(pk, pre["Xq"], spec)
    out["measured_peaks"] = mp
    out["roofline"]["frac_of_measured_mfma_peak"] = round(pre["tops_linear"] / mp["mfma_int8_tops"], 4)
    if not a.no_decode:
        d = bench_decode(L, pk)
        d["frac_of_measured_read_peak"] = d["gbs_hbm"] / mp["read_gbs_decode_size"]
        d["read_only_launch_gbs"] = mp["read_gbs_decode_size"]
        # can a call of this size reach 70 % of 8 TB/s at all?  A launch that only reads the same bytes says.
        d["target_0.70_reachable"] = bool(mp["read_gbs_decode_size"] >= 0.70 * HBM_PEAK_GBS)
        out["decode"] = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in d.items()}
        # the wide decode layer of configs[3] (W4A4, K=8192, N=28672: 125 MB per call), M = 1
        spec4 = workloads.config4(1)
        L4 = workloads.make_layer(spec4, want=("s", "W", "R"))
        pk4 = serq.pack_weights(L4["W"].to("cuda:0"), L4["s"].to("cuda:0"), 0, want_R=False, want_Rp=False)
        d4 = bench_decode(L4, pk4, reps=3, spec=spec4)
        stick4 = read_stick(int(decode_bytes(spec4)))
        d4["read_only_launch_gbs"] = stick4
        d4["frac_of_measured_read_peak"] = d4["gbs_hbm"] / stick4
        d4["target_0.70_reachable"] = bool(stick4 >= 0.70 * HBM_PEAK_GBS)
        out["decode_cfg4"] = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in d4.items()}
        del L4, pk4
    if not a.no_mx:
        # the MXFP4 variant of the same layer (its own line with `--mx`): step, layer kernel, quantiser
        mx = bench_mx(min(a.steps, 300), min(a.warmup, 30))
        out["mxfp4"] = {"step_tflops": mx["value"], "ms_per_step": mx["ms_per_step"],
                        "kernel": mx["roofline"]["kernel"], "kernel_ms": mx["roofline"]["kernel_ms"],
                        "kernel_tflops": mx["roofline"]["achieved"], "frac_of_fp4_peak": mx["roofline"]["frac"],
                        "frac_of_measured_mfma_peak": mx["roofline"]["frac_of_measured_mfma_peak"],
                        "mfma_fp4_tflops_measured": mx["measured_peaks"]["mfma_fp4_tflops"],
                        "quantize_act_ms": mx["quantize_act"]["ms"], "decode_M1_us": mx["decode"]["us_hbm"],
                        "decode_M1_gbs": mx["decode"]["gbs_hbm"]}
    if not a.no_cpu:
        cb, _ = cpu_baseline(L)
        cb["value"] = round(cb["value"], 5)
        out["cpu_baseline"] = cb
    print(json.dumps(out))


if __name__ == "__main__":
    main()
