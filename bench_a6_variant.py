#!/usr/bin/env python3
"""Head-to-head behind the library's 6-bit de-quantization: the same W6A16 kernels instantiated with the
chip's e3m2 -> fp16 conversion instruction (what the library ships) and with the shift/mask + exponent-bias
multiply of Section 5.3 of the paper on a bit arrangement made for it (bench_a6_variant.hip, bench only).

    python bench_a6_variant.py                 # builds libbench_a6_variant.so, checks equality, prints timings
    rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_MFMA SQ_VALU_MFMA_BUSY_CYCLES SQ_ACTIVE_INST_VALU SQ_WAVE_CYCLES \\
        --output-format csv -d out/a6 -o out -- python3 bench_a6_variant.py --profile

Both variants run the 8192 x 22016 layer at N = 16, 32 and 512 from graphs that rotate over 8 packed copies;
their outputs must be bit-identical (both de-quantizations are exact).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
SO = os.path.join(ROOT, "libbench_a6_variant.so")
SRC = os.path.join(ROOT, "bench_a6_variant.hip")


def build():
    deps = [SRC] + [os.path.join(ROOT, "paper_2401_14112_amd", "csrc", f)
                    for f in ("fp6_device.hpp", "linear_stream.hpp", "linear_tiled.hpp")]
    if os.path.exists(SO) and all(os.path.getmtime(d) <= os.path.getmtime(SO) for d in deps):
        return
    cmd = ["/opt/rocm/bin/hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", ROOT,
           SRC, "-o", SO]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode:
        raise RuntimeError("hipcc failed:\n" + r.stdout)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--profile", action="store_true", help="a few eager launches of each variant, for a profiler run")
    ap.add_argument("--N", type=str, default="16,32,512")
    args = ap.parse_args()
    build()
    import torch

    import paper_2401_14112_amd as pkg
    import workloads

    L = ctypes.CDLL(SO)
    vp, i64, ci, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    L.a6_workspace_bytes.restype = sz
    L.a6_workspace_bytes.argtypes = [i64, i64]
    L.a6_repack.restype = ci
    L.a6_repack.argtypes = [vp, vp, i64, i64, vp]
    L.a6_linear.restype = ci
    L.a6_linear.argtypes = [ci, vp, vp, vp, vp, i64, i64, i64, vp, vp]
    dev = "cuda:0"
    name, M, K = workloads.FFN_65B
    NB = 8
    packed, repacked, scales = [], [], []
    for b in range(NB):
        pk, sc = pkg.fp6_quantize_pack(workloads.make_weights(M, K, seed=b, device=dev))
        rp = torch.empty_like(pk)
        assert L.a6_repack(pk.data_ptr(), rp.data_ptr(), M, K, None) == 0
        packed.append(pk)
        repacked.append(rp)
        scales.append(sc)
    torch.cuda.synchronize()
    out = {}
    for N in [int(v) for v in args.N.split(",")]:
        X = workloads.make_activations(N, K, seed=N, device=dev)
        Y = [torch.empty((N, M), dtype=torch.float16, device=dev) for _ in range(2)]
        ws = torch.zeros(L.a6_workspace_bytes(M, N), dtype=torch.uint8, device=dev)

        def launch(variant, b, stream):
            w = (packed if variant == 0 else repacked)[b]
            rc = L.a6_linear(variant, w.data_ptr(), scales[b].data_ptr(), X.data_ptr(), Y[variant].data_ptr(), M, N, K,
                             ws.data_ptr(), stream)
            assert rc == 0, rc

        st = torch.cuda.current_stream().cuda_stream
        for variant in (0, 1):
            for b in range(NB):
                launch(variant, b, st)
        torch.cuda.synchronize()
        assert torch.equal(Y[0].view(torch.int16), Y[1].view(torch.int16)), "the two de-quantizations disagree"
        ref = pkg.fp6_linear(packed[NB - 1], scales[NB - 1], X, M, K)
        torch.cuda.synchronize()
        assert torch.equal(Y[0].view(torch.int16), ref.view(torch.int16)), "the bench build differs from the library"
        if args.profile:
            continue
        row = {}
        graphs = []
        for variant in (0, 1):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                cs = torch.cuda.current_stream().cuda_stream
                for i in range(32):
                    launch(variant, i % NB, cs)
            g.replay()
            g.replay()
            graphs.append(g)
        torch.cuda.synchronize()
        times = [[], []]
        for rnd in range(6):     # interleaved, so that both variants see the same machine state
            for variant in (0, 1):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                graphs[variant].replay()
                graphs[variant].replay()
                e1.record()
                torch.cuda.synchronize()
                times[variant].append(e0.elapsed_time(e1) * 1e3 / 64)
        for variant, label in ((0, "conversion_instruction"), (1, "shift_mask_eq3")):
            t = sorted(times[variant])
            row[label + "_us"] = round(t[len(t) // 2], 2)
        row["shift_mask_over_conversion"] = round(row["shift_mask_eq3_us"] / row["conversion_instruction_us"], 3)
        out[str(N)] = row
    print(json.dumps({"layer": name, "M": M, "K": K, "outputs_bit_identical": True, "per_n": out}))


if __name__ == "__main__":
    main()
