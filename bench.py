#!/usr/bin/env python3
"""Benchmark of the fused RMSNorm + MatMul hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload decode] [--variant auto]

A step is one rmsnorm_linear call (stage W and X, X (.) g, sum of squares, contraction, split-K
reduce, row scale, store) on one seeded synthetic batch.  The default workload is the decode
projection (X 1x4096, W 4096x4096, bf16), the HBM-bound configuration the headline metric is quoted
on; --workload selects another of the five configurations.  Inputs are resident in HBM before the
timed region.  So that a small W is not simply served from the 256 MB Infinity Cache, steps rotate
through enough distinct copies of (X, g, W, Y) to exceed 512 MiB; the same-buffer ("warm") rate is
reported beside it.  The K timed steps are enqueued as one HIP graph on the current stream and are
bracketed by HIP events on that stream, so elapsed / K approaches the kernel's own duration.

Prints ONE JSON line.  `roofline` prices the dominant kernel against the published MI355X peak;
`cpu_baseline` is the fp64 CPU oracle timed on this machine's host cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = 2500.0        # MI355X dense bf16/fp16 matrix, published (2.5 PFLOP/s)
MFMA_PEAK_TFLOPS_F32 = 157.3     # MI355X fp32 matrix, published


def mfma_peak(dtype):
    return MFMA_PEAK_TFLOPS_F32 if dtype == "f32" else MFMA_PEAK_TFLOPS
ROTATE_BYTES = 512 << 20
MIN_REGION_MS = 50.0             # a timed region is the K-step graph replayed until it lasts at least this long
# HBM-side bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs), scaled by what the same
# counters read for the plain copy kernel: profiles/hbm_traffic_pmc.md, which gives the commands.  Counters
# cannot be read from inside this process, so every figure is stored with the launch it was measured on
# (variant, columns per workgroup, K slabs, workgroups; rl_last_launch) and is reported only while the
# library still launches that shape; otherwise `traffic` is null.
MEASURED_TRAFFIC = {
    # workload: (bytes per launch = 2.0 x FETCH_SIZE + 1.0 x WRITE_SIZE in KiB x 1024, launch the counters were read on)
    "decode": (34.45e6, ("gemv", 128, 16, 512)),
    "qkv": (55.05e6, ("skinny", 128, 4, 192)),
    "gateup": (243.15e6, ("skinny", 128, 1, 224)),
    "prefill": (2035.9e6, ("tile_pre", 256, 8, 1024)),      # both kernels: 268.9 MB + 1767.0 MB
}
TRAFFIC_SOURCE = "profiles/hbm_traffic_pmc.md"


def _time_region(fn_enqueue, torch, min_ms=MIN_REGION_MS):
    """Events on the current stream around enough calls of fn_enqueue() (one call = one replay of the
    K-step graph) to last min_ms; returns (event ms per call, wall ms per call, calls)."""
    start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    fn_enqueue()
    end.record()
    torch.cuda.synchronize()
    once = max(start.elapsed_time(end), 1e-3)
    calls = max(1, min(2000, int(np.ceil(min_ms / once))))
    t0 = time.perf_counter()
    start.record()
    for _ in range(calls):
        fn_enqueue()
    end.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3
    return start.elapsed_time(end) / calls, wall / calls, calls


def _workload(name):
    """One of the five configurations by name, or "MxKxN" ("MxKxN:f32", ":f16"): a workload of that shape
    (same recipe), bf16 unless a type is named."""
    import workloads
    if name in workloads.CONFIG_NAMES:
        return workloads.config(name)
    shape, _, dtype = name.lower().partition(":")
    M, K, N = (int(v) for v in shape.split("x"))
    return workloads.make(M, K, N, dtype or "bf16", 1e-5, 4242 + M + K + N, name=name, outlier_frac=0.05,
                          n_check_rows=min(M, 64))


def run_workload(rl, torch, name, steps, warmup, variant, use_graph=True, check=True, gated=False, autotune=False,
                 interleaved=False, only_cold=False, ceilings=True):
    import workloads
    from tests.util import compare, compare_gated, to_device, to_host_f64

    w = _workload(name)
    tdt = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}[w.dtype]
    abytes = w.algorithmic_bytes
    NY = w.N // 2 if gated else w.N              # gated block: W = [gate | up], Y has H = N/2 columns
    if gated:
        abytes -= 2 * w.M * (w.N - NY)
    copies = max(1, min(steps, -(-ROTATE_BYTES // abytes)))
    if name == "prefill":
        copies = 2
    X0, g0, W0 = to_device(w.X, w.dtype), to_device(w.g, w.dtype), to_device(w.W, w.dtype)
    Xs, gs, Ws, Ys = [X0], [g0], [W0], [torch.empty((w.M, NY), dtype=tdt, device="cuda")]
    for _ in range(copies - 1):
        Xs.append(X0.clone()); gs.append(g0.clone()); Ws.append(W0.clone()); Ys.append(torch.empty_like(Ys[0]))

    rl.rl_set_variant(variant)
    fused_call = rl.rmsnorm_gated_mlp if gated else rl.rmsnorm_linear
    Wf = Ws                                      # what the fused call reads
    if gated and interleaved:                    # gate and up columns interleaved in groups of 64, repacked once
        fused_call = rl.rmsnorm_gated_mlp_interleaved
        Wf = [rl.rl_interleave_gate_up(W) for W in Ws]
    tuned = None
    if autotune:                                 # the library's search over launch shapes, on the rotating copies
        rl.rl_autotune_rotating(X0, g0, Wf, w.eps, Ys[0], gated=gated, interleaved=gated and interleaved, reps=3 * len(Wf))
        tuned = rl.rl_autotune_get(w.M, w.K, w.N, tdt, gated, gated and interleaved)

    def step(i):
        j = i % copies
        fused_call(Xs[j], gs[j], Wf[j], w.eps, Ys[j])

    for i in range(max(warmup, 1)):
        step(i)
    torch.cuda.synchronize()
    used = rl.rl_last_variant()

    def make_runner(step_fn):
        if use_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for i in range(steps):
                    step_fn(i)
            graph.replay()                       # one untimed replay
            torch.cuda.synchronize()
            return graph.replay
        return lambda: [step_fn(i) for i in range(steps)]

    cold = make_runner(step)
    ev_ms, wall_ms, replays = min((_time_region(cold, torch) for _ in range(3)), key=lambda t: t[0])
    launch = rl.rl_last_launch()                 # (variant, columns, slabs, workgroups) of the timed call
    if only_cold:
        per = ev_ms / steps
        return {"workload": name, "variant": used, "launch": launch, "us_per_step": per * 1e3, "replays": replays,
                "copies_rotated": copies, "algorithmic_bytes": abytes, "flops": w.flops}, w
    warm = make_runner(lambda i: fused_call(Xs[0], gs[0], Wf[0], w.eps, Ys[0]))
    warm_ms, _, _ = min((_time_region(warm, torch) for _ in range(3)), key=lambda t: t[0])

    # the unfused pair from the same library, same rotation, for the fusion gain on this hardware
    # (gated block: the fused norm + products followed by the separate activation kernel)
    Xn = [torch.empty_like(x) for x in Xs]
    Zs = [torch.empty((w.M, w.N), dtype=tdt, device="cuda") for _ in range(copies)] if gated else None

    def pair(i):
        j = i % copies
        if gated:
            rl.rmsnorm_linear(Xs[j], gs[j], Ws[j], w.eps, Zs[j])
            rl.silu_mul(Zs[j], Ys[j])
        else:
            rl.rmsnorm(Xs[j], gs[j], w.eps, Xn[j])
            rl.matmul(Xn[j], Ws[j], Ys[j])

    pair(0)
    torch.cuda.synchronize()
    pair_ms, _, _ = min((_time_region(make_runner(pair), torch) for _ in range(3)), key=lambda t: t[0])

    # where the automatic choice is the two-kernel tile form, the one fused kernel is timed beside it
    one_kernel_ms = None
    if used == "tile_pre" and variant == "auto":
        rl.rl_set_variant("tile")
        step(0)
        torch.cuda.synchronize()
        one_kernel_ms, _, _ = min((_time_region(make_runner(step), torch) for _ in range(3)), key=lambda t: t[0])
        rl.rl_set_variant("auto")

    parity = None
    if check:
        import oracle
        step(0)
        torch.cuda.synchronize()
        rows = torch.from_numpy(w.check_rows).cuda()
        Y = to_host_f64(Ys[0][rows], w.dtype)
        Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps, rows=w.check_rows)
        if gated:
            parity = compare_gated(Y, Z, w.dtype, name)      # largest err / bound (<= 1)
        else:
            parity, _ = compare(Y, Z, w.dtype, name)
    rl.rl_set_variant("auto")

    per_step_ms = ev_ms / steps
    mem_bound = w.M <= 64
    # what a bare read of the same W, launched and timed the same way, takes: the workgroups' own access shape
    # (256-byte strips, as many row parts as the launch has slabs) and one contiguous share per workgroup
    ceiling = None
    if ceilings and mem_bound and w.dtype != "f32" and (w.N * 2) % 256 == 0:
        sink = torch.zeros(4, dtype=torch.int32, device="cuda")
        parts = max(1, launch[2]) if launch[0] in ("gemv", "skinny") else 1
        wbytes = w.K * w.N * 2
        strips = make_runner(lambda i: rl.rl_probe_read_strips(Ws[i % copies], w.K, w.N * 2, parts, sink))
        t_strips, _, _ = min((_time_region(strips, torch) for _ in range(3)), key=lambda t: t[0])
        flat = make_runner(lambda i: rl.rl_probe_read_flat(Ws[i % copies], wbytes, 512, sink))
        t_flat, _, _ = min((_time_region(flat, torch) for _ in range(3)), key=lambda t: t[0])
        ceiling = {"what": "a bare read of W alone (no X, no product, no exchange between workgroups), same graph, rotation and events",
                   "strips_256B_us": t_strips / steps * 1e3, "strips_256B_GBps": wbytes / (t_strips / steps * 1e-3) / 1e9,
                   "strips_row_parts": parts,
                   "contiguous_us": t_flat / steps * 1e3, "contiguous_GBps": wbytes / (t_flat / steps * 1e-3) / 1e9}
    elif ceilings and not mem_bound and w.dtype != "f32":
        sink = torch.zeros(rl.lib().rl_probe_mfma_sink_floats(), dtype=torch.float32, device="cuda")
        fl = rl.rl_probe_mfma(sink, 2000, tdt)
        torch.cuda.synchronize()
        t_m, _, _ = min((_time_region(lambda: rl.rl_probe_mfma(sink, 2000, tdt), torch) for _ in range(3)), key=lambda t: t[0])
        t_m0, _, _ = min((_time_region(lambda: rl.rl_probe_mfma(sink, 2000, tdt, zero_operands=True), torch) for _ in range(3)),
                         key=lambda t: t[0])
        ceiling = {"what": "register-only 32x32x16 matrix-core loop on pseudo-random operands, nothing else; and the same loop on "
                           "zero operands (no switching activity: the clock the published peak assumes)",
                   "mfma_loop_TFLOPs": fl / (t_m * 1e-3) / 1e12, "mfma_loop_zero_operands_TFLOPs": fl / (t_m0 * 1e-3) / 1e12}
        # the same call on all-zero operands: same kernels, same launch, no switching activity in the
        # multipliers -- what the schedule delivers when the matrix cores' power draw does not lower the clock
        Xz, Wz = torch.zeros_like(X0), torch.zeros_like(W0)
        zero = make_runner(lambda i: fused_call(Xz, gs[0], Wz, w.eps, Ys[0]))
        t_z, _, _ = min((_time_region(zero, torch) for _ in range(3)), key=lambda t: t[0])
        ceiling["same_call_on_zero_operands_us"] = t_z / steps * 1e3
        ceiling["same_call_on_zero_operands_TFLOPs"] = w.flops / (t_z / steps * 1e-3) / 1e12
        del Xz, Wz
    res = {
        "workload": name + ("+gate" if gated else "") + ("(interleaved W)" if gated and interleaved else ""), "M": w.M, "K": w.K, "N": w.N, "dtype": w.dtype, "variant": used,
        "launch": {"variant": launch[0], "columns": launch[1], "slabs": launch[2], "workgroups": launch[3]},
        "copies_rotated": copies, "timed_replays_of_the_graph": replays, "us_per_step": per_step_ms * 1e3,
        "us_per_step_warm": warm_ms / steps * 1e3, "us_per_step_unfused_pair": pair_ms / steps * 1e3,
        "wall_us_per_step": wall_ms / steps * 1e3,
        "us_per_step_one_fused_kernel": None if one_kernel_ms is None else one_kernel_ms / steps * 1e3,
        "TBps": abytes / (per_step_ms * 1e-3) / 1e12, "TBps_warm": abytes / (warm_ms / steps * 1e-3) / 1e12,
        "TFLOPs": w.flops / (per_step_ms * 1e-3) / 1e12,
        "algorithmic_bytes": abytes, "flops": w.flops,
        "max_err_over_rmsY": parity, "autotuned": tuned, "measured_ceiling": ceiling,
    }
    rl.rl_autotune_clear()
    if mem_bound:
        res["roofline_frac"] = res["TBps"] * 1e3 / HBM_PEAK_GBS
    else:
        res["roofline_frac"] = res["TFLOPs"] / mfma_peak(w.dtype)
    return res, w


def run_ntrans(rl, torch, steps, warmup, M=16384, D=2048, dtype="bf16", with_cpu=True):
    """The nTrans chain y = Norm(x + alpha Norm(h - x)) on seeded rows of an nGPT-sized hidden state."""
    import oracle
    import workloads
    from tests.util import compare, to_device, to_host_f64
    rng = np.random.default_rng(240505751 + 11)
    x = workloads.to_storage(rng.standard_normal((M, D), dtype=np.float32), dtype)
    h = workloads.to_storage(rng.standard_normal((M, D), dtype=np.float32), dtype)
    a = workloads.to_storage((rng.uniform(0.0, 1.0, D) * 0.3).astype(np.float32), dtype)
    eps = float(np.float32(1e-6))
    abytes = 2 * (3 * M * D + D)
    copies = max(1, -(-ROTATE_BYTES // abytes))
    xs = [to_device(x, dtype)]; hs = [to_device(h, dtype)]; ad = to_device(a, dtype)
    for _ in range(copies - 1):
        xs.append(xs[0].clone()); hs.append(hs[0].clone())
    ys = [torch.empty_like(xs[0]) for _ in range(copies)]
    step = lambda i: rl.rl_ntrans(xs[i % copies], hs[i % copies], ad, eps, ys[i % copies])
    for i in range(max(warmup, 1)):
        step(i)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(steps):
            step(i)
    graph.replay(); torch.cuda.synchronize()
    ev_ms, _, _ = min((_time_region(graph.replay, torch) for _ in range(3)), key=lambda t: t[0])
    rows = np.arange(0, M, max(1, M // 64))
    Z = oracle.ntrans(x[rows], h[rows], a, dtype, eps)
    parity, _ = compare(to_host_f64(ys[0][torch.from_numpy(rows).cuda()], dtype), Z, dtype, "ntrans")
    us = ev_ms / steps * 1e3
    out = {"metric": "nTrans chain TB/s", "value": abytes / us / 1e6, "unit": "TB/s", "n_gpus": 1, "steps": steps,
           "warmup": warmup, "ms_per_step": us / 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": dtype, "data": "synthetic",
           "config": {"workload": f"ntrans: x, h {M}x{D}, alpha {D}, {dtype}", "copies_rotated": copies},
           "roofline": {"bound": "hbm", "achieved": abytes / us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": abytes / us / 1e3 / HBM_PEAK_GBS, "traffic": None, "kernel": "ntrans_vec_kernel",
                        "us_per_launch": us},
           "detail": {"us_per_step": us, "algorithmic_bytes": abytes, "max_err_over_rmsY": parity}}
    if with_cpu:
        n, t0, reps = min(M, 4096), time.perf_counter(), 0
        while time.perf_counter() - t0 < 10.0 and reps < 200:
            oracle.ntrans(x[:n], h[:n], a, dtype, eps); reps += 1
        sec = (time.perf_counter() - t0) / reps
        out["cpu_baseline"] = {"value": 2 * (3 * n * D + D) / sec / 1e12, "unit": "TB/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": f"{reps} run(s) of the fp64 oracle on {n} of {M} rows, {sec:.4f} s each"}
    return out


def run_qknorm(rl, torch, steps, warmup, B=8, H=32, S=4096, D=128, dtype="bf16", with_cpu=True):
    """QKNorm in front of attention, decode form, on a seeded key-value cache: 32 heads of 128, 4K
    context (the paper's QKNorm setting: Chameleon-7B's attention shape and context length)."""
    import oracle
    import workloads
    from tests.util import to_device, to_host_f64
    c = workloads.make_attention(B, H, S, D, dtype, 240505751 + 13)
    eps = float(np.float32(1e-5))
    abytes = 2 * (2 * B * H * S * D + 2 * B * H * D + 4 * D)
    copies = max(2, -(-(2 * ROTATE_BYTES) // abytes))   # at least 1 GiB of keys and values in rotation
    dev = {k: to_device(v, dtype) for k, v in c.items()}
    Ks = [dev["K"]] + [dev["K"].clone() for _ in range(copies - 1)]
    Vs = [dev["V"]] + [dev["V"].clone() for _ in range(copies - 1)]
    Os = [torch.empty_like(dev["Q"]) for _ in range(copies)]
    step = lambda i: rl.rl_qknorm_attention(dev["Q"], Ks[i % copies], Vs[i % copies], dev["gq"], dev["bq"],
                                            dev["gk"], dev["bk"], eps, Os[i % copies])
    for i in range(max(warmup, 1)):
        step(i)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(steps):
            step(i)
    graph.replay(); torch.cuda.synchronize()
    ev_ms, _, _ = min((_time_region(graph.replay, torch) for _ in range(3)), key=lambda t: t[0])
    us = ev_ms / steps * 1e3
    nb = min(B, 2)                                   # parity on the first samples
    want = oracle.qknorm_attention(c["Q"][:nb], c["K"][:nb], c["V"][:nb], c["gq"], c["bq"], c["gk"], c["bk"], dtype, eps)
    got = to_host_f64(Os[0][:nb].contiguous(), dtype)
    parity = float((np.abs(got - want).max(-1) / np.sqrt((want ** 2).mean(-1))).max())
    assert parity <= 2e-2, f"qknorm attention: max|err|/rms = {parity:.3e}"
    # the unfused baseline the paper describes (normalisation kernels, then an attention kernel), from the
    # vendor stack behind torch: for context only
    import torch.nn.functional as F
    def unfused():
        qn = F.layer_norm(dev["Q"], (D,), dev["gq"], dev["bq"], eps)
        kn = F.layer_norm(dev["K"], (D,), dev["gk"], dev["bk"], eps)
        return F.scaled_dot_product_attention(qn.unsqueeze(2), kn, dev["V"])
    for _ in range(3):
        unfused()
    torch.cuda.synchronize()
    t_ms, _, _ = min((_time_region(lambda: [unfused() for _ in range(10)], torch, min_ms=0.0) for _ in range(3)), key=lambda t: t[0])
    out = {"metric": "QKNorm + attention TB/s", "value": abytes / us / 1e6, "unit": "TB/s", "n_gpus": 1, "steps": steps,
           "warmup": warmup, "ms_per_step": us / 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": dtype, "data": "synthetic",
           "config": {"workload": f"qknorm: Q {B}x{H}x{D}, K and V {B}x{H}x{S}x{D}, {dtype}", "copies_rotated": copies},
           "roofline": {"bound": "hbm", "achieved": abytes / us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": abytes / us / 1e3 / HBM_PEAK_GBS, "traffic": None,
                        "kernel": "qkattn_kernel",
                        "us_per_launch": us},
           "detail": {"us_per_step": us, "algorithmic_bytes": abytes, "max_err_over_rms": parity,
                      "us_per_step_torch_unfused_one_buffer": t_ms / 10 * 1e3}}
    if with_cpu:
        t0, reps = time.perf_counter(), 0
        while time.perf_counter() - t0 < 10.0 and reps < 200:
            oracle.qknorm_attention(c["Q"][:1], c["K"][:1], c["V"][:1], c["gq"], c["bq"], c["gk"], c["bk"], dtype, eps)
            reps += 1
        sec = (time.perf_counter() - t0) / reps
        out["cpu_baseline"] = {"value": abytes / B / sec / 1e12, "unit": "TB/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": f"{reps} run(s) of the fp64 oracle on 1 of {B} samples, {sec:.4f} s each"}
    return out


def probe_strips(rl, torch, spec):
    """Finish times of the workgroups of rl_probe_read_strips (one per 256-byte strip), by address class."""
    shape, _, shift = spec.partition("+")
    rows, row_bytes = (int(v) for v in shape.lower().split("x"))
    shift = int(shift or 0)
    strips = row_bytes // 256
    nbytes = rows * row_bytes
    copies = max(2, -(-ROTATE_BYTES // nbytes))
    pool = torch.randint(0, 1 << 30, ((copies * nbytes + shift) // 4 + 64,), dtype=torch.int32, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    slots = rl.rl_trace_slots()
    buf = torch.zeros(strips * slots, dtype=torch.int64, device="cuda")
    src = lambda i: pool.view(torch.uint8)[shift + (i % copies) * nbytes:][:nbytes]
    for i in range(4):
        rl.rl_probe_read_strips(src(i), rows, row_bytes, 1, sink)
    torch.cuda.synchronize()
    rl.rl_set_trace(buf)
    sums, count = np.zeros(4), np.zeros(4)
    last = 0.0
    try:
        for i in range(8):
            buf.zero_()
            s = src(i)
            rl.rl_probe_read_strips(s, rows, row_bytes, 1, sink)
            torch.cuda.synchronize()
            t = buf.cpu().numpy().reshape(-1, slots).astype(np.float64)
            fin = (t[:, 2] - t[:, 0].min()) * 10.0                      # ns after the first workgroup started
            b = np.arange(strips)
            strip = (b % 8) * (strips // 8) + b // 8 if strips % 8 == 0 else b
            cls = ((s.data_ptr() + strip * 256) >> 8) & 3
            for c in range(4):
                sums[c] += fin[cls == c].sum(); count[c] += (cls == c).sum()
            last += fin.max() / 8
    finally:
        rl.rl_set_trace(None)
    return {"probe": "rl_probe_read_strips, one workgroup per 256-byte strip", "rows": rows, "row_bytes": row_bytes,
            "base_shift": shift, "workgroups": strips, "last_finish_ns": last,
            "mean_finish_ns_by_address_bits_9_8": {f"{c:02b}": (sums[c] / count[c] if count[c] else None) for c in range(4)}}


def cpu_baseline(w, mem_bound, budget_s=12.0):
    """The oracle as it stands, on the host cores, on a bounded sample of the same workload."""
    import oracle
    rows = w.check_rows if w.M > 64 else np.arange(w.M)
    reps, t_total = 0, 0.0
    t_start = time.perf_counter()
    while True:
        t0 = time.perf_counter()
        oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps, rows=rows)
        t_total += time.perf_counter() - t0
        reps += 1
        if time.perf_counter() - t_start > budget_s or reps >= 5000:
            break
    sec = t_total / reps
    frac = len(rows) / w.M
    if mem_bound:
        value, unit = w.algorithmic_bytes / sec / 1e12, "TB/s"
    else:
        value, unit = 2.0 * len(rows) * w.K * w.N / sec / 1e12, "TFLOP/s"
    return {"value": value, "unit": unit, "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{reps} run(s) of the fp64 oracle on {len(rows)} of {w.M} rows "
                      f"({frac:.3g} of the workload), {sec:.3f} s each",
            "seconds_per_run": sec}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="decode",
                    help="decode, tiny, qkv, gateup, prefill, ntrans, qknorm (batch 8; qknorm1, qknorm16; a head "
                         "size other than 128 as qknorm:64 or qknorm1:256), "
                         "or MxKxN (a bf16 workload of that shape; MxKxN:f32 or :f16 for another type)")
    ap.add_argument("--variant", default="auto")
    ap.add_argument("--no-graph", action="store_true", help="enqueue the timed steps one by one")
    ap.add_argument("--others", action="store_true", help="(default) also time the other four configurations")
    ap.add_argument("--no-others", action="store_true", help="time the named workload only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU baseline leg")
    ap.add_argument("--autotune", action="store_true",
                    help="let the library's launch-shape tuner pick the shape for this workload first")
    ap.add_argument("--interleaved", action="store_true",
                    help="with --gated: W's gate and up columns interleaved in groups of 64 (rmsnorm_gated_mlp_interleaved)")
    ap.add_argument("--gated", action="store_true",
                    help="time the gated block (SiLU(gate) * up epilogue, W read as [gate | up]) on the workload")
    ap.add_argument("--only-cold", action="store_true",
                    help="time the rotating-buffer graph of the named workload only (for a kernel trace of one phase)")
    ap.add_argument("--probe-strips", default="", metavar="ROWSxROW_BYTES[+SHIFT]",
                    help="only read a matrix of that shape as 256-byte column strips, one workgroup each, and report "
                         "when the strips finish, by bits [9:8] of their first byte's address (SHIFT bytes added to the base)")
    ap.add_argument("--probe-copy", type=int, default=0, metavar="MiB",
                    help="only run the plain copy kernel on MiB of data ten times (memory-counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (a split of W and Y along N across GPUs needs no exchange; it is not built here)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    import paper_2405_05751_amd as rl
    rl.lib()                                      # fail loudly if the HIP library is not built

    if args.probe_copy:
        n = args.probe_copy << 20
        src = torch.randint(0, 1 << 30, (n // 4,), dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            rl.rl_probe_copy(dst, src)
        torch.cuda.synchronize()
        print(json.dumps({"probe_copy_bytes_read": n, "probe_copy_bytes_written": n, "launches": 10}))
        return

    if args.probe_strips:
        print(json.dumps(probe_strips(rl, torch, args.probe_strips)))
        return

    name = args.workload
    if name == "ntrans":
        print(json.dumps(run_ntrans(rl, torch, args.steps if args.steps is not None else 100, args.warmup,
                                    with_cpu=not args.no_cpu)))
        return
    if name.split(":")[0] in ("qknorm", "qknorm1", "qknorm16"):
        B = {"qknorm": 8, "qknorm1": 1, "qknorm16": 16}[name.split(":")[0]]
        D = int(name.split(":")[1]) if ":" in name else 128
        print(json.dumps(run_qknorm(rl, torch, args.steps if args.steps is not None else 100, args.warmup, B=B, D=D,
                                    with_cpu=not args.no_cpu)))
        return
    steps = args.steps if args.steps is not None else (20 if name == "prefill" else 200)
    if args.steps is None and "x" in name and name != "prefill":
        M, K, N = (int(v) for v in name.lower().partition(":")[0].split("x"))
        steps = 20 if 2.0 * M * K * N > (1e10 if name.lower().endswith(":f32") else 2e11) else 100
    res, w = run_workload(rl, torch, name, steps, args.warmup, args.variant, use_graph=not args.no_graph,
                          gated=args.gated, autotune=args.autotune, interleaved=args.interleaved,
                          only_cold=args.only_cold)
    if args.only_cold:
        print(json.dumps(res))
        return
    out = headline(name, res, w, steps, args)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, w.M <= 64)
    if (args.others or name == "decode") and not args.no_others:
        import workloads
        others = []
        for other in workloads.CONFIG_NAMES:
            if other == name:
                continue
            r, wo = run_workload(rl, torch, other, 20 if other == "prefill" else 200, args.warmup, args.variant,
                                 use_graph=not args.no_graph)
            r["roofline"] = roofline_of(other, r, wo, args.variant == "auto")
            others.append(r)
        # the fp32 path (the decode projection's shape, and a matrix-bound one) on its own kernel
        for other, st in (("1x4096x4096:f32", 200), ("2048x4096x4096:f32", 20)):
            r, wo = run_workload(rl, torch, other, st, args.warmup, args.variant, use_graph=not args.no_graph, ceilings=False)
            r["roofline"] = roofline_of(other, r, wo, False)
            others.append(r)
        # the widened rows of the path, each with its own roofline (no CPU leg: the headline carries one)
        r, wo = run_workload(rl, torch, "gateup", 200, args.warmup, args.variant, use_graph=not args.no_graph,
                             gated=True, interleaved=True, ceilings=False)
        r["roofline"] = roofline_of("gateup+gate", r, wo, False)
        others.append(r)
        others.append(run_ntrans(rl, torch, 100, args.warmup, with_cpu=False))
        others.append(run_qknorm(rl, torch, 100, args.warmup, B=8, with_cpu=False))
        others.append(run_qknorm(rl, torch, 100, args.warmup, B=1, with_cpu=False))
        out["other_workloads"] = others
    print(json.dumps(out))


def roofline_of(name, res, w, auto):
    """The roofline object of one workload's dominant kernel."""
    if w.M <= 64:
        roof = {"bound": "hbm", "achieved": res["TBps"] * 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    else:
        roof = {"bound": "mfma", "achieved": res["TFLOPs"], "peak": mfma_peak(w.dtype), "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    launch = [res["launch"][k] for k in ("variant", "columns", "slabs", "workgroups")]
    rec = MEASURED_TRAFFIC.get(name)
    if auto and rec is not None and list(rec[1]) == launch:
        roof["traffic"] = rec[0]
        roof["traffic_source"] = f"{TRAFFIC_SOURCE}: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE on this launch shape {launch}"
    else:
        roof["traffic"] = None
        roof["traffic_source"] = ("not measured for the launch shape of this run " + str(launch) if rec is not None
                                  else "not measured for this workload")
    roof["kernel"] = res["variant"]
    roof["us_per_launch"] = res["us_per_step"]
    if res.get("measured_ceiling"):
        roof["measured_ceiling"] = res["measured_ceiling"]
    if res.get("us_per_step_one_fused_kernel"):
        # the automatic choice at this size is two kernels (X-hat written once, then the product); the
        # one fused kernel is timed beside it and priced the same way
        one = res["us_per_step_one_fused_kernel"]
        roof["form"] = "two kernels: X-hat and 1/rms written once by a first kernel, then the tile product scaled per row"
        roof["one_fused_kernel"] = {"us_per_launch": one, "achieved": w.flops / one / 1e6, "frac": w.flops / one / 1e6 / mfma_peak(w.dtype)}
    return roof


def headline(name, res, w, steps, args):
    mem_bound = w.M <= 64
    if mem_bound:
        metric, unit, value = "fused RMSNorm+MatMul TB/s", "TB/s", res["TBps"]
    else:
        metric, unit, value = "fused RMSNorm+MatMul TFLOP/s", "TFLOP/s", res["TFLOPs"]
    roof = roofline_of(name + ("+gate" if args.gated else ""), res, w, args.variant == "auto" and not args.gated)
    return {
        "metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": res["us_per_step"] / 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{name}{' + gate' if args.gated else ''}: X {w.M}x{w.K}, W {w.K}x{w.N}, {w.dtype}",
                   "variant": res["variant"], "launch": res["launch"],
                   "copies_rotated": res["copies_rotated"], "graph": not args.no_graph,
                   "timed_region": f"the {steps}-step graph replayed {res['timed_replays_of_the_graph']} times between two events "
                                   f"(at least {MIN_REGION_MS:.0f} ms); ms_per_step = events / (replays x steps)"},
        "roofline": roof,
        "detail": res,
    }


if __name__ == "__main__":
    main()
