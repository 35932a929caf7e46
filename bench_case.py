#!/usr/bin/env python3
"""Runs fp6_linear (or fp6g_linear, fp5_linear, fp4_linear, fp3_linear, fp16_linear) at one shape and a list of token
counts a few times on cuda:0 and prints the time per launch.

Meant to be the program of a profiler run, e.g.

    rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES GRBM_GUI_ACTIVE -- python3 bench_case.py --N 32,64,512

Every token count runs a different kernel instantiation (16-, 32-, 64-token streaming kernels, the tiled
kernel's block shapes), so the dispatches of one run are told apart by kernel name.  Weights are synthetic
(N(0, 0.02) rounded to fp16, quantized by fp6_quantize_pack); every launch reads another of `--buffers`
packed copies so that the weights come from HBM, not from the last-level cache.

    python3 bench_case.py --M 512 --N 512 --tile 256x128 --split 1   # a pinned block shape and split-K factor: with
                                         # S = 1 every block does all K/256 k-tiles, so M sets how many CUs are busy
    python3 bench_case.py --chain80      # the 80-GEMM decoder chain of bench.py alone (one graph; with and without
                                         # a branch that reads ahead in the next layer's weights)
"""
from __future__ import annotations

import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--M", type=int, default=8192)
    ap.add_argument("--K", type=int, default=22016)
    ap.add_argument("--N", type=str, default="512", help="token counts, comma separated")
    ap.add_argument("--reps", type=int, default=16)
    ap.add_argument("--buffers", type=int, default=8)
    ap.add_argument("--which", choices=("fp6", "fp6g", "fp5", "fp4", "fp3", "fp16"), default="fp6")
    ap.add_argument("--tile", type=str, default="", help="force the block of the tiled kernel, e.g. 256x128 (rows x tokens)")
    ap.add_argument("--split", type=int, default=0, help="force the split-K factor (0 = automatic)")
    ap.add_argument("--chain80", action="store_true",
                    help="instead: the 80 GEMMs of 20 decoder blocks of a 70B-class model from one HIP graph, plain and "
                         "with a second graph branch that reads half of the next layer's weights (bench.py's measurement)")
    args = ap.parse_args()

    import torch

    import paper_2401_14112_amd as pkg
    import workloads

    pkg.load_library()
    dev = "cuda:0"
    if args.chain80:
        import json

        import numpy as np

        import bench

        out = bench.decoder_set_measurements(pkg, torch, np, workloads, dev)
        print(json.dumps(out["weight_stream_80_gemms_one_graph"]), flush=True)
        return
    M, K = args.M, args.K
    if args.tile:
        rows, tokens = (int(v) for v in args.tile.split("x"))
        pkg.fp6_tuning_set_tile(rows, tokens)
    pkg.fp6_tuning_set_split_k(args.split)
    weights = []
    for b in range(args.buffers):
        W = workloads.make_weights(M, K, seed=b, device=dev)
        weights.append((W,) if args.which == "fp16" else getattr(pkg, args.which + "_quantize_pack")(W))
    query = getattr(pkg, ("fp6" if args.which == "fp6g" else args.which) + "_linear_workspace_bytes")
    for N in [int(v) for v in args.N.split(",")]:
        X = workloads.make_activations(N, K, seed=N, device=dev)
        Y = torch.empty((N, M), dtype=torch.float16, device=dev)
        ws = torch.zeros(max(query(M, N, K), 16), dtype=torch.uint8, device=dev)

        def launch(i):
            w = weights[i % len(weights)]
            if args.which == "fp6g":
                pkg.fp6g_linear(w[0], w[1], X, M, K, 128, out=Y, workspace=ws)
            elif args.which != "fp16":
                getattr(pkg, args.which + "_linear")(w[0], w[1], X, M, K, out=Y, workspace=ws)
            else:
                pkg.fp16_linear(w[0], X, out=Y, workspace=ws)

        for i in range(4):
            launch(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(args.reps):
            launch(i)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / args.reps
        print("%s_linear M=%d K=%d N=%d: %.2f us per launch (eager, %d launches), %.1f TFLOP/s" % (
            args.which, M, K, N, us, args.reps, 2.0 * M * N * K / us * 1e-6), flush=True)


if __name__ == "__main__":
    main()
