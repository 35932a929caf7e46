#!/usr/bin/env python3
"""Benchmark of the W6A16 linear layer on one MI355X.

Workload (the paper's Fig. 1 layer, llama-65b FFN, W = 8192 x 22016, batch swept): one
"step" is the decode sweep N = 1, 2, 4, 8, 16, 32 of fp6_linear over packed e3m2 weights,
i.e. six launches of the runtime path (weight fetch, activation staging, register unpack,
MFMA contraction, split-K reduction, scaled epilogue).  Every launch reads a different one
of 8 packed copies of the layer (1.08 GB in total) so that no weight byte is served from
the 256 MB last-level cache.  The ahead-of-time steps (fp6_quantize_pack) and the test aid
(fp6_unpack) are timed once each outside the step and reported under "offline".

Prints ONE JSON line.  `value` = packed weight bytes streamed per second over the timed
steps (whole job, launches replayed from captured HIP graphs); `roofline` prices the
dominant kernel (the 16-token streaming kernel) with HIP events recorded around at least ten
replays of a graph of its launches, and carries the rest of the metric inside it: `per_n`
(every N = 1 ... 512: microseconds per launch and the fraction of the HBM and of the
matrix-core roof) and `mfma` (the tiled kernel at N = 512 against the 2.5 PFLOP/s roof);
`cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E, vendor figure
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense fp16 matrix peak, vendor figure
N_BUFFERS = 8


def device_record(torch):
    """What the runtime reports about the device the figures were measured on (clocks are the maxima it
    advertises; the peaks used for the fractions are the vendor's figures above)."""
    p = torch.cuda.get_device_properties(0)
    rec = {"name": p.name, "compute_units": p.multi_processor_count, "memory_GiB": round(p.total_memory / 2 ** 30, 1)}
    for key, attr in (("max_engine_clock_MHz", "clock_rate"), ("max_memory_clock_MHz", "memory_clock_rate")):
        v = getattr(p, attr, None)
        if v:
            rec[key] = round(v / 1000.0, 1)
    for key, attr in (("memory_bus_bits", "memory_bus_width"), ("l2_bytes", "L2_cache_size"), ("gcn_arch", "gcnArchName")):
        v = getattr(p, attr, None)
        if v:
            rec[key] = v
    return rec


def algorithmic_bytes(M, N, K):
    """Bytes one fp6_linear call must move: packed weights + scales once, X once, Y once."""
    return 3 * M * K // 4 + 2 * M + 2 * K * N + 2 * M * N


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the prefill / fp16 / offline side measurements")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the layer is a single-GPU kernel and nothing here "
              "uses a second GPU); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2401_14112_amd as pkg
    import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    pkg.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    name, M, K = workloads.FFN_65B
    sweep = list(workloads.DECODE_N)
    P = pkg.fp6_packed_bytes(M, K)

    # ---- inputs resident in HBM: 8 packed copies of the layer (different seeds), activations per N
    packed, scales = [], []
    pack_ms = []
    W0 = None
    for b in range(N_BUFFERS):
        W = workloads.make_weights(M, K, seed=b, device=dev)
        pk = torch.empty(P, dtype=torch.uint8, device=dev)
        sc = torch.empty(M, dtype=torch.float16, device=dev)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        pkg.fp6_quantize_pack(W, pk, sc)
        e1.record()
        torch.cuda.synchronize()
        pack_ms.append(e0.elapsed_time(e1))
        packed.append(pk)
        scales.append(sc)
        if b == 0:
            W0 = W
        else:
            del W
    Xs = {n: workloads.make_activations(n, K, seed=n, device=dev) for n in sweep}
    Ys = {n: torch.empty((n, M), dtype=torch.float16, device=dev) for n in sweep}
    ws_bytes = max(pkg.fp6_linear_workspace_bytes(M, n, K) for n in sweep)
    ws = torch.zeros(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    def launch(n, b):
        pkg.fp6_linear(packed[b], scales[b], Xs[n], M, K, out=Ys[n], workspace=ws)

    # the rotation (launch j reads buffer j % 8) repeats every 4 steps of 6 launches
    period = 1
    while (period * len(sweep)) % N_BUFFERS:
        period += 1
    for n in sweep:          # first launches outside any capture
        launch(n, 0)
    torch.cuda.synchronize()
    graphs = []
    for s in range(period):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i, n in enumerate(sweep):
                launch(n, (s * len(sweep) + i) % N_BUFFERS)
        graphs.append(g)
    # `period` consecutive steps (one pass over the rotation) as ONE graph: a graph launch has a fixed cost
    # that a serving loop would also spread over as many launches as it can capture
    rotation = torch.cuda.CUDAGraph()
    with torch.cuda.graph(rotation):
        for s in range(period):
            for i, n in enumerate(sweep):
                launch(n, (s * len(sweep) + i) % N_BUFFERS)
    # and LONG rotations as one graph (the fixed cost of a graph launch is ~20 us on this runtime: over 24
    # launches that is most of a microsecond each)
    LONG = 5
    long_rotation = torch.cuda.CUDAGraph()
    with torch.cuda.graph(long_rotation):
        for r in range(LONG):
            for s in range(period):
                for i, n in enumerate(sweep):
                    launch(n, (s * len(sweep) + i) % N_BUFFERS)

    # ---- quick validity check of what is being timed (sampled rows against the CPU oracle)
    from oracle import fp6_oracle as oracle
    tiles = np.array([0, 37, M // 16 - 1])
    rows = (tiles[:, None] * 16 + np.arange(16)[None, :]).ravel()
    # tiles are stored k-tile major: the stream of the sub-matrix of the listed row tiles is, per k-tile, their bytes
    sub_packed = packed[0].view(K // 256, M // 16, 3072)[:, torch.from_numpy(tiles).to(dev), :].reshape(-1).cpu().numpy()
    sub_scales = scales[0].cpu().numpy()[rows]
    worst = 0.0
    for n in (1, 32):
        launch(n, 0)
        torch.cuda.synchronize()
        ref = oracle.linear(sub_packed, sub_scales, Xs[n].cpu().numpy(), len(rows), K)
        got = Ys[n].cpu().numpy()[:, rows].astype(np.float64)
        worst = max(worst, float((np.abs(got - ref).max(axis=1) / (5e-3 * np.abs(ref).max(axis=1))).max()))
    if worst > 1.0:
        print("bench.py: fp6_linear disagrees with the oracle (error/bound = %.3g)" % worst, file=sys.stderr)
        sys.exit(3)

    # a plain copy of known size: the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this same
    # command are scaled by what they read for this kernel (512 MiB read, 512 MiB written)
    cal_src = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    # ---- timed region: W warm-up steps, then exactly K steps between synchronizations
    def run_steps(count):
        """Exactly `count` steps: LONG rotations at a time from the long graph, then whole rotations, the
        remainder from single-step graphs."""
        for _ in range(count // (period * LONG)):
            long_rotation.replay()
        count %= period * LONG
        for _ in range(count // period):
            rotation.replay()
        for s in range(count % period):
            graphs[s].replay()

    # every graph that the timed region replays is replayed twice first (a graph's first replay carries
    # one-off costs), then the W warm-up steps proper
    for g in [long_rotation, rotation] + graphs:
        g.replay()
        g.replay()
    run_steps(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(args.steps)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    step_weight_bytes = P * len(sweep)
    step_flops = sum(2.0 * M * n * K for n in sweep)
    value_gbps = step_weight_bytes / (ms_per_step * 1e-3) * 1e-9

    # ---- per-N durations with HIP events on the launch stream, same steps launched eagerly (each figure
    # includes the launch gap and the two event records)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(sweep) + 1)] for _ in range(args.steps)]
    j = 0
    torch.cuda.synchronize()
    for s in range(args.steps):
        ev[s][0].record()
        for i, n in enumerate(sweep):
            launch(n, j % N_BUFFERS)
            j += 1
            ev[s][i + 1].record()
    torch.cuda.synchronize()
    per_n_us = {}
    for i, n in enumerate(sweep):
        d = np.array([ev[s][i].elapsed_time(ev[s][i + 1]) for s in range(args.steps)]) * 1e3
        per_n_us[n] = (float(d.mean()), float(np.median(d)), float(d.min()))
    # ... and from graphs of 64 launches of one N over the rotation of weight copies: the kernel's own pace
    graph_us = {n: _time_graph(torch, lambda i, n=n: launch(n, i % N_BUFFERS), N_BUFFERS, reps=24, min_launches=64) for n in sweep}
    # ---- the dominant kernel (the 16-token streaming kernel: the N <= 16 launches of a step) on its own:
    # the same launches with the same buffer rotation, captured without the N = 32 launch, HIP events on the
    # launch stream around every replay; duration per launch = elapsed / launches in the replay
    small = [n for n in sweep if n <= 16]
    dom_graph = torch.cuda.CUDAGraph()
    DOM_PASSES = 3
    with torch.cuda.graph(dom_graph):
        for r in range(DOM_PASSES):
            for s in range(period):
                for i, n in enumerate(sweep):
                    if n <= 16:
                        launch(n, (s * len(sweep) + i) % N_BUFFERS)
    for s in range(max(2, args.warmup // period)):
        dom_graph.replay()
    # one pair of events brackets one replay of the whole rotation (an event record is a stream operation of
    # its own and would otherwise add its gap to every five launches); at least ten replays whatever --steps is
    groups = max(10, args.steps // (period * DOM_PASSES))
    dev_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(groups)]
    torch.cuda.synchronize()
    for gi in range(groups):
        dev_ev[gi][0].record()
        dom_graph.replay()
        dev_ev[gi][1].record()
    torch.cuda.synchronize()
    dom_us_all = np.array([a.elapsed_time(b) for a, b in dev_ev]) * 1e3 / (len(small) * period * DOM_PASSES)
    dom_bytes = sum(algorithmic_bytes(M, n, K) for n in small) / len(small)
    dom_us = float(dom_us_all.mean())
    achieved = dom_bytes / (dom_us * 1e-6) * 1e-9

    # ---- the prefill half of the metric (N = 64 ... 512) and the compute-bound roofline: every N from a graph
    # of one launch per weight copy, HIP events around each of >= 10 replays
    prefill = {}
    for n in workloads.PREFILL_N:
        Xp = workloads.make_activations(n, K, seed=n, device=dev)
        Yp = torch.empty((n, M), dtype=torch.float16, device=dev)
        wsp = torch.zeros(max(pkg.fp6_linear_workspace_bytes(M, n, K), 16), dtype=torch.uint8, device=dev)
        prefill[n] = _time_graph_stats(
            torch, np, lambda i: pkg.fp6_linear(packed[i % N_BUFFERS], scales[i % N_BUFFERS], Xp, M, K, out=Yp, workspace=wsp),
            N_BUFFERS, replays=10)
        del Xp, Yp, wsp
    per_n = {}
    for n in sweep:
        per_n[str(n)] = _per_n_entry(M, n, K, graph_us[n])
    for n in workloads.PREFILL_N:
        per_n[str(n)] = _per_n_entry(M, n, K, prefill[n]["mean_us"])
    n_mfma = max(workloads.PREFILL_N)
    mfma_tflops = 2.0 * M * n_mfma * K / prefill[n_mfma]["mean_us"] * 1e-6

    result = {
        "metric": "W6A16 GEMM effective weight GB/s + TFLOP/s, 8192x22016, N=1..512",
        "value": round(value_gbps, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",   # the matrix instructions take fp16 operands (weights de-quantized from e3m2) and add in fp32
        "data": "synthetic",
        "config": {
            "workload": "llama65b_ffn W[8192x22016] W6A16 linear, one step = decode sweep N in "
                        "{1,2,4,8,16,32}, launch j reads packed copy j mod 8 (1.08 GB rotation), replayed from HIP graphs of %d steps" % (period * LONG),
            "M": M, "K": K, "N_sweep": sweep, "weight_buffers": N_BUFFERS,
            "layout_version": pkg.fp6_layout_version(),
            "arithmetic": "e3m2 weights de-quantized to f16 in registers x f16 activations, f32 accumulate, one f16 rounding",
        },
        "device": device_record(torch),
        "tflops": round(step_flops / (ms_per_step * 1e-3) * 1e-12, 2),
        "roofline": {
            "bound": "hbm",
            "kernel": "linear_stream_kernel<PackedFp6Source, NT=1> (N <= 16 launches of the step)",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": read_traffic_profile(),
            "algorithmic_bytes_per_launch": int(dom_bytes),
            "avg_launch_us": round(dom_us, 2),
            "min_launch_us": round(float(dom_us_all.min()), 2),
            "max_launch_us": round(float(dom_us_all.max()), 2),
            "replays_timed": int(groups),
            "launches_per_replay": len(small) * period * DOM_PASSES,
            # the compute-bound half: the tiled kernel at the largest N of the metric against the matrix-core roof
            "mfma": {
                "bound": "mfma", "kernel": "linear_tiled_kernel<PackedFp6Source> at N = %d" % n_mfma,
                "achieved": round(mfma_tflops, 1), "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(mfma_tflops / MFMA_F16_PEAK_TFLOPS, 4), "flops_per_launch": 2 * M * n_mfma * K,
                "avg_launch_us": round(prefill[n_mfma]["mean_us"], 2), "min_launch_us": round(prefill[n_mfma]["min_us"], 2),
                "replays_timed": prefill[n_mfma]["replays"], "launches_per_replay": N_BUFFERS,
            },
            # every N of the metric: microseconds per launch (graph replay) and the fraction of each roof
            "per_n": per_n,
            "min_hbm_frac_N_le_32": min(per_n[str(n)]["hbm_frac"] for n in sweep),
            # all launches of the timed step together (N = 32 included): their algorithmic bytes over the step time
            "whole_step_hbm_frac": round(sum(algorithmic_bytes(M, n, K) for n in sweep) / (ms_per_step * 1e-3) * 1e-9
                                         / HBM_PEAK_GBPS, 4),
            "timing": "HIP events around each replay of a graph of the N<=16 launches of %d steps, elapsed/%d"
                      % (period * DOM_PASSES, len(small) * period * DOM_PASSES),
        },
        "sweep": {
            str(n): {
                "us": round(graph_us[n], 2),      # per launch, graph replay
                "weight_GBps": round(P / graph_us[n] * 1e-3, 1),
                "tflops": round(2.0 * M * n * K / graph_us[n] * 1e-6, 2),
                "hbm_frac": round(algorithmic_bytes(M, n, K) / graph_us[n] * 1e-3 / HBM_PEAK_GBPS, 4),
                # launched one by one with an event record after each (the host's launch pace and the records' gaps included)
                "eager_us_mean": round(per_n_us[n][0], 2), "eager_us_median": round(per_n_us[n][1], 2),
                "eager_us_min": round(per_n_us[n][2], 2),
            } for n in sweep
        },
        "oracle_check_err_over_bound": round(worst, 4),
    }

    if not args.no_extras:
        result["offline"] = side_measurements(pkg, torch, np, workloads, M, K, W0, packed, scales, pack_ms)
        ceil = result["offline"]["empirical_ceilings"]
        result["roofline"]["measured_peak_GBps"] = ceil["read_stream_1GiB_GBps"]
        result["roofline"]["frac_of_measured_peak"] = round(achieved / ceil["read_stream_1GiB_GBps"], 4)
        result["roofline"]["frac_of_same_size_read_stream"] = round(
            ceil["read_stream_one_launch_135MB_us"] / dom_us, 4)
    del W0

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(oracle, np, workloads, packed[0], scales[0], M, K, sweep)

    # the long side measurements go last, so that a reader that keeps only the head of the line keeps the contract
    if "offline" in result:
        result["offline"] = result.pop("offline")
    print(json.dumps(result))


def read_traffic_profile():
    """HBM bytes per launch of the dominant kernel, measured by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
    this command and scaled by the calibration copy; read from the committed summary if it is there."""
    path = os.path.join(ROOT, "profiles", "fp6_linear_stream_decode_8192x22016_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return int(float(line.split(":")[1].split()[0]))
    except OSError:
        pass
    return None


def _per_n_entry(M, n, K, us):
    tfl = 2.0 * M * n * K / us * 1e-6
    return {"us": round(us, 2), "hbm_frac": round(algorithmic_bytes(M, n, K) / us * 1e-3 / HBM_PEAK_GBPS, 4),
            "mfma_frac": round(tfl / MFMA_F16_PEAK_TFLOPS, 4)}


def _time_graph_stats(torch, np, fn, launches_per_graph, replays=10):
    """Microseconds per launch of fn(i), i in range(launches_per_graph), captured as one graph that is warmed
    twice and then replayed `replays` times with a pair of HIP events around each replay."""
    fn(0)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(launches_per_graph):
            fn(i)
    g.replay()
    g.replay()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(replays)]
    for a, b in ev:
        a.record()
        g.replay()
        b.record()
    torch.cuda.synchronize()
    us = np.array([a.elapsed_time(b) for a, b in ev]) * 1e3 / launches_per_graph
    return {"mean_us": float(us.mean()), "min_us": float(us.min()), "replays": replays}


def _time_graph(torch, fn, launches_per_graph, reps=20, min_launches=24):
    """Average microseconds per launch of fn(i) for i in range(launches_per_graph), from graph replays.  The
    graph holds as many passes over those launches as it takes to reach min_launches, so that the fixed cost of
    a graph launch is spread the same way for every kernel that is compared."""
    fn(0)
    torch.cuda.synchronize()
    passes = max(1, -(-min_launches // launches_per_graph))
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(passes):
            for i in range(launches_per_graph):
                fn(i)
    g.replay()
    torch.cuda.synchronize()
    reps = max(2, -(-reps // passes))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (reps * passes * launches_per_graph)


def _compare_sweep(pkg, torch, workloads, M, K, packed, scales, W16, Ns):
    """fp6_linear against the library's own fp16_linear (and, as context, the vendor fp16 GEMM torch dispatches
    to) at the same shapes; every launch of a graph reads another copy of the weights."""
    dev = packed[0].device
    P = pkg.fp6_packed_bytes(M, K)
    cmp = {}
    for n in Ns:
        X = workloads.make_activations(n, K, seed=n, device=dev)
        Y = torch.empty((n, M), dtype=torch.float16, device=dev)
        ws6 = torch.zeros(max(pkg.fp6_linear_workspace_bytes(M, n, K), 16), dtype=torch.uint8, device=dev)
        ws16 = torch.zeros(max(pkg.fp16_linear_workspace_bytes(M, n, K), 16), dtype=torch.uint8, device=dev)
        reps = 10 if n <= 32 else 3
        us6 = _time_graph(torch, lambda i: pkg.fp6_linear(packed[i % len(packed)], scales[i % len(packed)], X, M, K, out=Y, workspace=ws6), len(packed), reps)
        us16 = _time_graph(torch, lambda i: pkg.fp16_linear(W16[i % len(W16)], X, out=Y, workspace=ws16), len(W16), reps)
        try:
            usv = round(_time_graph(torch, lambda i: torch.matmul(X, W16[i % len(W16)].t(), out=Y), len(W16), reps), 2)
        except Exception:      # the vendor path is context only; never let it break the benchmark
            usv = None
        tfl = 2.0 * M * n * K / us6 * 1e-6
        cmp[str(n)] = {"fp6_us": round(us6, 2), "fp16_us": round(us16, 2), "speedup_vs_own_fp16": round(us16 / us6, 3),
                       "vendor_fp16_gemm_us": usv,
                       "fp6_weight_GBps": round(P / us6 * 1e-3, 1), "fp6_tflops": round(tfl, 2),
                       "fp6_hbm_frac": round(algorithmic_bytes(M, n, K) / us6 * 1e-3 / HBM_PEAK_GBPS, 4),
                       "fp6_mfma_frac": round(tfl / MFMA_F16_PEAK_TFLOPS, 4)}
    return cmp


def side_measurements(pkg, torch, np, workloads, M, K, W0, packed, scales, pack_ms):
    """Prefill-sized N, the library's own fp16 GEMM at the same shapes, the offline steps, the transposed
    (down-projection) shape, and the 70B-class layer set / decoder weight stream."""
    dev = W0.device
    P = pkg.fp6_packed_bytes(M, K)
    out = {"quantize_pack_ms": round(float(np.median(pack_ms)), 3),
           "quantize_pack_GBps_fp16_read": round(2.0 * M * K / (float(np.median(pack_ms)) * 1e-3) * 1e-9, 1)}
    Wd = torch.empty((M, K), dtype=torch.float16, device=dev)
    us = _time_graph(torch, lambda i: pkg.fp6_unpack(packed[i % len(packed)], scales[i % len(packed)], M, K, out=Wd), 4, reps=5)
    out["unpack_ms"] = round(us * 1e-3, 3)
    out["unpack_GBps_total"] = round((P + 2.0 * M * K) / us * 1e-3, 1)
    del Wd
    # the same launch with the weights resident in the last-level cache (one packed copy, 135 MB): labelled
    # as such, never the headline
    X1 = workloads.make_activations(1, K, seed=1, device=dev)
    Y1 = torch.empty((1, M), dtype=torch.float16, device=dev)
    ws1 = torch.zeros(max(pkg.fp6_linear_workspace_bytes(M, 1, K), 16), dtype=torch.uint8, device=dev)
    us = _time_graph(torch, lambda i: pkg.fp6_linear(packed[0], scales[0], X1, M, K, out=Y1, workspace=ws1), 8, reps=10)
    out["cache_resident_N1_us"] = round(us, 2)
    # the library's own W16A16 kernel on 3 fp16 copies (1.08 GB rotation)
    W16 = [W0] + [workloads.make_weights(M, K, seed=100 + b, device=dev) for b in range(2)]
    Ns = list(workloads.DECODE_N) + list(workloads.PREFILL_N)
    out["vs_own_fp16_linear"] = _compare_sweep(pkg, torch, workloads, M, K, packed, scales, W16, Ns)
    # the transposed shape (down projection, 22016 x 8192): the same bytes seen as [K][M] are a valid input
    Mt, Kt = K, M
    W16t = [w.view(Mt, Kt) for w in W16]
    pk_t, sc_t = [], []
    for b in range(len(packed)):
        Wt = W16t[b] if b < len(W16t) else workloads.make_weights(Mt, Kt, seed=200 + b, device=dev)
        pk, sc = pkg.fp6_quantize_pack(Wt)
        pk_t.append(pk)
        sc_t.append(sc)
        del Wt
    out["down_projection_22016x8192"] = _compare_sweep(pkg, torch, workloads, Mt, Kt, pk_t, sc_t, W16t, Ns)
    out["w5a16_e2m2"] = narrow_sweep(pkg, "fp5", torch, workloads, M, K, W16, Ns)
    out["w4a16_e2m1"] = narrow_sweep(pkg, "fp4", torch, workloads, M, K, W16, Ns)
    out["w3a16_e2m0"] = narrow_sweep(pkg, "fp3", torch, workloads, M, K, W16, Ns)
    out["w6a16_group128"] = narrow_sweep(pkg, "fp6g", torch, workloads, M, K, W16, Ns)
    del W16, W16t, pk_t, sc_t
    torch.cuda.empty_cache()
    out["decoder_set_70b"] = decoder_set_measurements(pkg, torch, np, workloads, dev)
    out["fused_feed_forward_70b"] = fused_block_measurements(pkg, torch, workloads, dev)
    out["model_blocks_vs_fp16"] = model_block_measurements(pkg, torch, workloads, dev)
    out["empirical_ceilings"] = empirical_ceilings(pkg, torch, packed)
    out["independent_chains"] = independent_chain_measurements(pkg, torch, workloads, M, K, packed, scales)
    return out


def narrow_sweep(pkg, prefix, torch, workloads, M, K, W16, Ns):
    """Another weight format (prefix "fp5": e2m2, 5MK/8 bytes; "fp4": e2m1, MK/2 bytes; "fp3": e2m0, 3MK/8 bytes; "fp6g": e3m2 with a scale
    per row and 128 columns) on the same layer:
    its linear call at every N, rotating over 8 packed copies, plus its quantize_pack and unpack once."""
    dev = W16[0].device
    if prefix == "fp6g":      # e3m2 codes, one scale per row and 128 columns (extra 2MK/128 bytes of scales)
        packed_bytes, workspace_bytes = pkg.fp6_packed_bytes, pkg.fp6_linear_workspace_bytes
        quantize_pack = lambda W, pk, sc: pkg.fp6g_quantize_pack(W, 128, pk, sc)
        unpack = lambda pk, sc, M, K, out: pkg.fp6g_unpack(pk, sc, M, K, 128, out=out)
        linear = lambda pk, sc, X, M, K, out, workspace: pkg.fp6g_linear(pk, sc, X, M, K, 128, out=out, workspace=workspace)
        n_scales = M * (K // 128)
    else:
        packed_bytes = getattr(pkg, prefix + "_packed_bytes")
        quantize_pack = getattr(pkg, prefix + "_quantize_pack")
        unpack = getattr(pkg, prefix + "_unpack")
        linear = getattr(pkg, prefix + "_linear")
        workspace_bytes = getattr(pkg, prefix + "_linear_workspace_bytes")
        n_scales = M
    P = packed_bytes(M, K)
    packed, scales, pack_ms = [], [], []
    for b in range(N_BUFFERS):
        W = W16[b] if b < len(W16) else workloads.make_weights(M, K, seed=300 + b, device=dev)
        pk = torch.empty(P, dtype=torch.uint8, device=dev)
        sc = torch.empty(n_scales, dtype=torch.float16, device=dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        quantize_pack(W, pk, sc)
        e1.record()
        torch.cuda.synchronize()
        pack_ms.append(e0.elapsed_time(e1))
        packed.append(pk)
        scales.append(sc)
        del W
    out = {"packed_bytes": P, "quantize_pack_ms": round(sorted(pack_ms)[len(pack_ms) // 2], 3)}
    Wd = torch.empty((M, K), dtype=torch.float16, device=dev)
    us = _time_graph(torch, lambda i: unpack(packed[i % len(packed)], scales[i % len(packed)], M, K, out=Wd), 4, reps=5)
    out["unpack_ms"] = round(us * 1e-3, 3)
    del Wd
    per_n = {}
    for n in Ns:
        X = workloads.make_activations(n, K, seed=n, device=dev)
        Y = torch.empty((n, M), dtype=torch.float16, device=dev)
        ws = torch.zeros(max(workspace_bytes(M, n, K), 16), dtype=torch.uint8, device=dev)
        us = _time_graph(torch, lambda i: linear(packed[i % len(packed)], scales[i % len(packed)], X, M, K, out=Y, workspace=ws),
                         len(packed), 10 if n <= 32 else 3)
        alg = P + 2 * n_scales + 2 * K * n + 2 * M * n
        tfl = 2.0 * M * n * K / us * 1e-6
        per_n[str(n)] = {"us": round(us, 2), "weight_GBps": round(P / us * 1e-3, 1), "tflops": round(tfl, 2),
                         "hbm_frac": round(alg / us * 1e-3 / HBM_PEAK_GBPS, 4), "mfma_frac": round(tfl / MFMA_F16_PEAK_TFLOPS, 4)}
    out["linear"] = per_n
    return out


def decoder_set_measurements(pkg, torch, np, workloads, dev, blocks=20):
    """The four linear layers of a 70B-class decoder block: each shape at N = 16 (rotating over the 20 packed
    copies), then 20 blocks x 4 layers = 80 GEMMs with weights of their own from ONE captured HIP graph at
    N = 1 and N = 32, and fp6_quantize_pack of all 80 weight matrices timed by events."""
    shapes = workloads.SET_70B
    packed = {name: [] for name, _, _ in shapes}
    scales = {name: [] for name, _, _ in shapes}
    pack_ms, pack_bytes = 0.0, 0.0
    for b in range(blocks):
        for j, (name, M, K) in enumerate(shapes):
            W = workloads.make_weights(M, K, seed=1000 + 4 * b + j, device=dev)
            pk = torch.empty(pkg.fp6_packed_bytes(M, K), dtype=torch.uint8, device=dev)
            sc = torch.empty(M, dtype=torch.float16, device=dev)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            pkg.fp6_quantize_pack(W, pk, sc)
            e1.record()
            torch.cuda.synchronize()
            if b > 0:                       # block 0 is the warm-up
                pack_ms += e0.elapsed_time(e1)
                pack_bytes += 2.0 * M * K
            packed[name].append(pk)
            scales[name].append(sc)
            del W
    out = {"quantize_pack_all_layers": {"matrices": (blocks - 1) * len(shapes), "ms_total": round(pack_ms, 2),
                                        "GBps_fp16_read": round(pack_bytes / pack_ms * 1e-6, 1)}}
    per_shape = {}
    for name, M, K in shapes:
        n = 16
        X = workloads.make_activations(n, K, seed=n, device=dev)
        Y = torch.empty((n, M), dtype=torch.float16, device=dev)
        ws = torch.zeros(max(pkg.fp6_linear_workspace_bytes(M, n, K), 16), dtype=torch.uint8, device=dev)
        us = _time_graph(torch, lambda i: pkg.fp6_linear(packed[name][i], scales[name][i], X, M, K, out=Y, workspace=ws), blocks, reps=5)
        per_shape[name] = {"M": M, "K": K, "N": n, "us": round(us, 2),
                           "weight_GBps": round(pkg.fp6_packed_bytes(M, K) / us * 1e-3, 1),
                           "tflops": round(2.0 * M * n * K / us * 1e-6, 2),
                           "hbm_frac": round(algorithmic_bytes(M, n, K) / us * 1e-3 / HBM_PEAK_GBPS, 4)}
    out["N16"] = per_shape
    stream = {}
    total_packed = sum(pkg.fp6_packed_bytes(M, K) for _, M, K in shapes) * blocks
    for n in (1, 32):
        Xs = {name: workloads.make_activations(n, K, seed=n, device=dev) for name, M, K in shapes}
        Ys = {name: torch.empty((n, M), dtype=torch.float16, device=dev) for name, M, K in shapes}
        wss = {name: torch.zeros(max(pkg.fp6_linear_workspace_bytes(M, n, K), 16), dtype=torch.uint8, device=dev)
               for name, M, K in shapes}

        def one(i):
            name, M, K = shapes[i % len(shapes)]
            b = i // len(shapes)
            pkg.fp6_linear(packed[name][b], scales[name][b], Xs[name], M, K, out=Ys[name], workspace=wss[name])

        us = _time_graph(torch, one, blocks * len(shapes), reps=5)
        gemms = blocks * len(shapes)
        alg = sum(algorithmic_bytes(M, n, K) for _, M, K in shapes) * blocks
        stream[str(n)] = {"gemms_per_graph": gemms, "ms_per_replay": round(us * gemms * 1e-3, 3),
                          "us_per_gemm": round(us, 2),
                          "weight_GBps": round(total_packed / (us * gemms) * 1e-3, 1),
                          "hbm_frac": round(alg / (us * gemms) * 1e-3 / HBM_PEAK_GBPS, 4)}
        # The same 80 launches with a second branch in the graph that reads the first half of layer i+1's
        # packed weights (the read probe, which computes nothing) while layer i runs: does warming the
        # last-level cache for the next layer shorten the chain?
        ref = {name: Ys[name].clone() for name in Ys}
        sink = torch.empty(1024, dtype=torch.int32, device=dev)
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            main = torch.cuda.current_stream()
            for i in range(gemms):
                if i + 1 < gemms:
                    side.wait_stream(main)      # the branch for layer i+1 starts when layer i-1 has finished
                    with torch.cuda.stream(side):
                        name, M, K = shapes[(i + 1) % len(shapes)]
                        buf = packed[name][(i + 1) // len(shapes)]
                        nb = (buf.numel() // 2) // (1 << 24) * (1 << 24)
                        if nb:
                            pkg.fp6_probe_read(buf[:nb], sink)
                one(i)
            main.wait_stream(side)
        g.replay()
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        us_b = e0.elapsed_time(e1) * 1e3 / (5 * gemms)
        stream[str(n)]["with_next_layer_read_branch"] = {
            "us_per_gemm": round(us_b, 2), "hbm_frac": round(alg / (us_b * gemms) * 1e-3 / HBM_PEAK_GBPS, 4),
            "outputs_equal": bool(all(torch.equal(ref[k].view(torch.int16), Ys[k].view(torch.int16)) for k in ref))}
        del g
    out["weight_stream_80_gemms_one_graph"] = stream
    return out


def fused_block_measurements(pkg, torch, workloads, dev, copies=4):
    """The feed-forward block of a 70B-class decoder (hidden 8192, inner 28672) as two launches of
    fp6_linear_fused - gate and up interleaved row by row with silu(gate) * up in the kernel, then the down
    projection adding into the residual stream in place - against the same block from fp6_linear plus
    separate element-wise kernels (torch's), from graphs that rotate over `copies` sets of weights."""
    F, H = 28672, 8192
    gu, dn = [], []
    for c in range(copies):
        W = workloads.make_weights(2 * F, H, seed=2000 + c, device=dev)
        gu.append(pkg.fp6_quantize_pack(W))
        del W
        W = workloads.make_weights(H, F, seed=2100 + c, device=dev)
        dn.append(pkg.fp6_quantize_pack(W))
        del W
    out = {"packed_bytes_per_block": pkg.fp6_packed_bytes(2 * F, H) + pkg.fp6_packed_bytes(H, F)}
    for n in (1, 16, 32):
        X = workloads.make_activations(n, H, seed=n, device=dev)
        G = torch.empty((n, 2 * F), dtype=torch.float16, device=dev)
        A = torch.empty((n, F), dtype=torch.float16, device=dev)
        T = torch.empty((n, F), dtype=torch.float16, device=dev)
        D = torch.empty((n, H), dtype=torch.float16, device=dev)
        R = torch.zeros((n, H), dtype=torch.float16, device=dev)
        ws1 = torch.zeros(max(pkg.fp6_linear_workspace_bytes(2 * F, n, H), 16), dtype=torch.uint8, device=dev)
        ws2 = torch.zeros(max(pkg.fp6_linear_workspace_bytes(H, n, F), 16), dtype=torch.uint8, device=dev)

        def fused(i):
            pkg.fp6_linear_fused(gu[i][0], gu[i][1], X, 2 * F, H, gated=True, out=A, workspace=ws1)
            pkg.fp6_linear_fused(dn[i][0], dn[i][1], A, H, F, residual=R, out=R, workspace=ws2)

        def separate(i):
            # the same arithmetic from the plain layer: the row order of the weights does not matter for the time
            pkg.fp6_linear(gu[i][0], gu[i][1], X, 2 * F, H, out=G, workspace=ws1)
            torch.sigmoid(G[:, 0::2], out=T)
            T.mul_(G[:, 0::2]).mul_(G[:, 1::2])
            pkg.fp6_linear(dn[i][0], dn[i][1], T, H, F, out=D, workspace=ws2)
            R.add_(D)

        us_f = _time_graph(torch, fused, copies, reps=5)
        R.zero_()
        us_s = _time_graph(torch, separate, copies, reps=5)
        alg = algorithmic_bytes(2 * F, n, H) - n * F * 2 + algorithmic_bytes(H, n, F) + n * H * 2
        out[str(n)] = {"fused_us_per_block": round(us_f, 2), "separate_us_per_block": round(us_s, 2),
                       "speedup": round(us_s / us_f, 3),
                       "fused_hbm_frac": round(alg / us_f * 1e-3 / HBM_PEAK_GBPS, 4)}
    return out


def independent_chain_measurements(pkg, torch, workloads, M, K, packed, scales):
    """Throughput when independent calls are available (two requests being decoded, the experts of a layer):
    48 calls of fp6_linear on the benchmark layer, rotating over the packed copies, captured as one chain on
    one stream and as two or three chains side by side on streams of their own (each chain with its own
    output and workspace).  A launch spends 4-5 us of its 24 outside its stream of weights (prologue, split-K
    epilogue, the spread between its waves); side by side the chains fill those for each other."""
    dev = packed[0].device
    calls = 48
    out = {}
    for n in (1, 16):
        X = workloads.make_activations(n, K, seed=n, device=dev)
        ws_bytes = max(pkg.fp6_linear_workspace_bytes(M, n, K), 16)
        Ys = [torch.empty((n, M), dtype=torch.float16, device=dev) for _ in range(3)]
        wss = [torch.zeros(ws_bytes, dtype=torch.uint8, device=dev) for _ in range(3)]

        def launch(b, chain):
            pkg.fp6_linear(packed[b % len(packed)], scales[b % len(packed)], X, M, K, out=Ys[chain], workspace=wss[chain])

        for b in range(len(packed)):
            launch(b, b % 3)
        torch.cuda.synchronize()
        row = {}
        for chains in (1, 2, 3):
            g = torch.cuda.CUDAGraph()
            sides = [torch.cuda.Stream() for _ in range(chains - 1)]
            with torch.cuda.graph(g):
                main = torch.cuda.current_stream()
                for st in sides:
                    st.wait_stream(main)
                for c in range(chains):
                    with torch.cuda.stream(main if c == 0 else sides[c - 1]):
                        for b in range(c, calls, chains):
                            launch(b, c)
                for st in sides:
                    main.wait_stream(st)
            for _ in range(3):
                g.replay()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(8):
                g.replay()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 8 / calls
            row["chains_%d" % chains] = {"us_per_call": round(us, 2),
                                         "weight_GBps": round(3 * M * K // 4 / us * 1e-3, 1),
                                         "hbm_frac": round(algorithmic_bytes(M, n, K) / us * 1e-3 / HBM_PEAK_GBPS, 4)}
            del g
        out[str(n)] = row
    return out


def empirical_ceilings(pkg, torch, packed):
    """What this device delivers to the request patterns of the linear kernels, measured in the same run: a
    read-only stream (the weight path's loads, nothing computed) over 1 GiB and over buffers of one launch's
    size (the packed copies of the benchmark layer, rotating), and a loop of matrix instructions on register
    operands.  The fractions in the sweep tables are against the vendor peaks; these are the measured ones."""
    dev = packed[0].device
    big = torch.empty(1 << 30, dtype=torch.uint8, device=dev).zero_()
    rsink = torch.empty(1024, dtype=torch.int32, device=dev)
    n_big = pkg.fp6_probe_read(big, rsink)
    us_big = _time_graph(torch, lambda i: pkg.fp6_probe_read(big, rsink), 4, reps=8)
    n_one = pkg.fp6_probe_read(packed[0], rsink)
    us_one = _time_graph(torch, lambda i: pkg.fp6_probe_read(packed[i % len(packed)], rsink), len(packed), reps=10)
    del big
    sink = torch.empty(4 << 20, dtype=torch.uint8, device=dev)
    iters = 5000
    flop = pkg.fp6_probe_mfma(iters, sink)
    us_mfma = _time_graph(torch, lambda i: pkg.fp6_probe_mfma(iters, sink), 2, reps=4)
    return {"read_stream_1GiB_GBps": round(n_big / us_big * 1e-3, 1),
            "read_stream_one_launch_135MB_us": round(us_one, 2),
            "read_stream_one_launch_135MB_GBps": round(n_one / us_one * 1e-3, 1),
            "mfma_f16_32x32x16_TFLOPs": round(flop / us_mfma * 1e-6, 1),
            # 256 CUs x 4 SIMDs, 32768 flop per instruction, one instruction per 32 clocks and SIMD at full rate
            "engine_clock_GHz_implied_by_the_matrix_loop": round(flop / us_mfma * 1e-6 / (1024 * 1024) * 1e3, 3)}


def model_block_measurements(pkg, torch, workloads, dev):
    """The experiment of the paper's Section 7.1 re-run inside this library: the four linear layers of one
    decoder block of LLaMA-7b/13b/33b/65b and OPT-30b/66b/175b (synthetic weights of those shapes) at batch 8, 16
    and 32, fp6_linear against the library's own fp16_linear and (context) the vendor fp16 GEMM.  Every layer is
    timed from a graph that rotates over enough copies of its weights to exceed the 256 MB last-level cache;
    reported per model: microseconds per block (sum over the four layers) and the speed-up over fp16."""
    out = {}
    for name, hidden, inner, gated in workloads.MODEL_DIMS:
        per_n = {str(n): {"fp6_us": 0.0, "fp16_us": 0.0, "vendor_fp16_us": 0.0} for n in (8, 16, 32)}
        for lname, M, K in workloads.model_layers(hidden, inner, gated):
            P = pkg.fp6_packed_bytes(M, K)
            copies = max(2, min(64, -(-600 * 1024 * 1024 // P)))
            copies16 = max(2, min(copies, -(-600 * 1024 * 1024 // (2 * M * K))))
            packed, W16 = [], []
            for c in range(copies):
                W = workloads.make_weights(M, K, seed=3000 + c, device=dev)
                packed.append(pkg.fp6_quantize_pack(W))
                if c < copies16:
                    W16.append(W)
                del W
            for n in (8, 16, 32):
                X = workloads.make_activations(n, K, seed=n, device=dev)
                Y = torch.empty((n, M), dtype=torch.float16, device=dev)
                ws6 = torch.zeros(max(pkg.fp6_linear_workspace_bytes(M, n, K), 16), dtype=torch.uint8, device=dev)
                ws16 = torch.zeros(max(pkg.fp16_linear_workspace_bytes(M, n, K), 16), dtype=torch.uint8, device=dev)
                r = per_n[str(n)]
                r["fp6_us"] += _time_graph(torch, lambda i: pkg.fp6_linear(packed[i][0], packed[i][1], X, M, K, out=Y, workspace=ws6), copies, reps=5)
                r["fp16_us"] += _time_graph(torch, lambda i: pkg.fp16_linear(W16[i], X, out=Y, workspace=ws16), copies16, reps=5)
                try:
                    r["vendor_fp16_us"] += _time_graph(torch, lambda i: torch.matmul(X, W16[i].t(), out=Y), copies16, reps=5)
                except Exception:      # context only
                    r["vendor_fp16_us"] = float("nan")
            del packed, W16
        block_bytes = sum(pkg.fp6_packed_bytes(M, K) for _, M, K in workloads.model_layers(hidden, inner, gated))
        for n, r in per_n.items():
            r["speedup_vs_own_fp16"] = round(r["fp16_us"] / r["fp6_us"], 3)
            r["speedup_vs_vendor_fp16"] = round(r["vendor_fp16_us"] / r["fp6_us"], 3)
            r["weight_GBps"] = round(block_bytes / r["fp6_us"] * 1e-3, 1)
            for k in ("fp6_us", "fp16_us", "vendor_fp16_us"):
                r[k] = round(r[k], 2)
        out[name] = {"packed_bytes_per_block": block_bytes, "batch": per_n}
    return out


def cpu_baseline(oracle, np, workloads, packed0, scales0, M, K, sweep):
    """The CPU oracle, as it stands, on the same layer over the same sweep, repeated until about 10 s of
    host time have been spent."""
    rows_n = M
    sub_packed = packed0.cpu().numpy()
    sub_scales = scales0[:rows_n].cpu().numpy()
    Xs = [workloads.make_activations(n, K, seed=n).numpy() for n in sweep]
    passes = 0
    t0 = time.perf_counter()
    while True:
        for X in Xs:
            oracle.linear(sub_packed, sub_scales, X, rows_n, K)
        passes += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or passes >= 16:
            break
    bytes_done = passes * len(sweep) * (rows_n * K * 3 // 4)
    return {
        "value": round(bytes_done / dt * 1e-9, 4),
        "unit": "GB/s",
        "cores": oracle.threads(),
        "kind": "oracle",
        "sample": "fp64 oracle.linear on all 8192 rows of the same 8192x22016 layer, %d passes of the same sweep "
                  "N in {1,2,4,8,16,32} (%.1f s); effective packed-weight bytes per second" % (passes, dt),
        "gflops": round(passes * sum(2.0 * rows_n * n * K for n in sweep) / dt * 1e-9, 2),
    }


if __name__ == "__main__":
    main()
