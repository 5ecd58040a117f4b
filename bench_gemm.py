#!/usr/bin/env python3
"""The four projections of one layer as single GEMM operations (gllm_op_gemm_bf16 / _splitk with the planner's tile
and split), weights rotating through HBM so that they are never cache-resident, in a sustained loop.

    python bench_gemm.py [--config llama3_8b_pp4] [--rows T] [--seconds S] [--only gate_up_swiglu]

Prints one JSON line: TFLOP/s per projection (HIP events around a run of launches of that projection alone) and the
sustained figure of the mixed loop (wall clock over S seconds).  The sustained loop is what a power or clock reading
taken beside it refers to, e.g.  `python bench_gemm.py --seconds 10 & sleep 5; amd-smi metric -p -c`
(profiles/gemm_power_and_clock.txt).
"""
import argparse
import json
import time

import torch

from paper_2504_14775_amd import binding as B
from paper_2504_14775_amd import synth


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="llama3_8b_pp4")
    ap.add_argument("--rows", type=int, default=2048)
    ap.add_argument("--seconds", type=float, default=5.0)
    ap.add_argument("--only", default="", help="one of qkv, o, gate_up_swiglu, down: only this projection in the loop")
    args = ap.parse_args()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    shape = synth.SHAPES[args.config]
    T, H, I = args.rows, shape.hidden, shape.intermediate
    pad = lambda v, q: (v + q - 1) // q * q
    n_qkv = pad((shape.n_q_heads + 2 * shape.n_kv_heads) * shape.head_dim, 256)
    q_dim = shape.n_q_heads * shape.head_dim
    Tp = pad(T, 256)
    # name -> (n, k, mode, max splits)
    problems = {"qkv": (n_qkv, H, B.GEMM_STORE_F32, 8), "o": (pad(H, 256), q_dim, B.GEMM_STORE_F32, 8),
                "gate_up_swiglu": (2 * pad(I, 128), H, B.GEMM_SWIGLU_BF16, 1), "down": (pad(H, 256), pad(I, 128), B.GEMM_STORE_F32, 8)}
    if args.only:
        problems = {args.only: problems[args.only]}
    runs = {}
    for name, (n, k, mode, ms) in problems.items():
        tile, splits = B.gllm_op_gemm_plan(T, n, k, mode, ms)
        copies = max(2, int(600e6 // (n * k * 2)) + 1)
        a = torch.randn(Tp, k, device=dev).to(torch.bfloat16)
        # random values: the buffers are read as the tiled weight layout, which for a random matrix is a random matrix
        ws = [(torch.randn(n, k, device=dev) * 0.02).to(torch.bfloat16) for _ in range(copies)]
        if mode == B.GEMM_SWIGLU_BF16:
            out = torch.zeros(T, n // 2, device=dev, dtype=torch.bfloat16)
            fn = lambda w, a=a, out=out, n=n, k=k, tile=tile: B.gllm_op_gemm_bf16(a, w, out, T, n, k, B.GEMM_SWIGLU_BF16, tile)
        else:
            out = torch.zeros(splits, T, n, device=dev, dtype=torch.float32)
            fn = lambda w, a=a, out=out, n=n, k=k, tile=tile, splits=splits: B.gllm_op_gemm_bf16_splitk(a, w, out, T, n, k, tile, splits)
        runs[name] = (fn, ws, 2.0 * T * n * k, tile, splits)
    result = {}
    for name, (fn, ws, flop, tile, splits) in runs.items():
        for w in ws:
            fn(w)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            for w in ws:
                fn(w)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / (3 * len(ws))
        result[name] = {"tile": tile, "splits": splits, "us": round(ms * 1e3, 1), "tflops": round(flop / ms / 1e9, 1)}
    # the sustained, mixed loop
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    done, i = 0.0, 0
    while time.perf_counter() - t0 < args.seconds:
        for _ in range(20):
            for name, (fn, ws, flop, _, _) in runs.items():
                fn(ws[i % len(ws)])
                done += flop
            i += 1
        torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    print(json.dumps({"metric": "bf16 GEMM throughput, the four projections of a layer, cold weights", "unit": "TFLOP/s",
                      "value": round(done / wall / 1e12, 1), "peak": 2500.0, "frac": round(done / wall / 2.5e15, 4),
                      "config": {"workload": args.config, "rows": T, "seconds": args.seconds}, "data": "synthetic", "dtype": "bf16",
                      "by_projection": result}))


if __name__ == "__main__":
    main()
