#!/usr/bin/env python3
"""Times the last-stage extras (include/gllm_head.h) on one GPU: final norm + vocabulary projection of the rows that
receive a token, and the sampler.  Shapes: the Llama-3-8B-shaped head (hidden 4096, vocabulary 128256) with the 257
rows of the benchmark batch of bench.py (256 decode rows + the row that ends the prefill chunk).

    python bench_head.py [--rows M] [--steps K] [--warmup W] [--no-cpu-baseline]

Prints one JSON line.  `value` = rows (sequences) that get a next token per second through projection + sampling.
roofline: the projection streams the vocabulary matrix once per call (vocab x hidden x 2 bytes, the algorithmic
bytes) -- with a few hundred rows it is HBM-bound, so `achieved` is GB/s against the 8 TB/s peak.
"""
import argparse
import json
import time

import numpy as np
import torch

from paper_2504_14775_amd import head as HD
from paper_2504_14775_amd import synth


def timed(fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--rows", type=int, default=257)
    ap.add_argument("--hidden", type=int, default=4096)
    ap.add_argument("--vocab", type=int, default=128256)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    H, V, M = args.hidden, args.vocab, args.rows
    T = 2048
    gain = synth.normal_bf16(0, 1, 0, H, 0.1, 1.0, device=dev)
    w = synth.normal_bf16(0, 2, 0, V * H, 0.02, 0.0, device=dev).view(V, H)
    x = torch.randn(T, H, device=dev, generator=torch.Generator(device=dev).manual_seed(0)) * 3.0
    rows = torch.arange(T - M, T, dtype=torch.int32, device=dev)
    head = HD.Head(H, V, M, 1e-6, device=dev)
    head.load(gain, w)
    logits = torch.empty(M, head.padded_vocab, dtype=torch.float32, device=dev)
    temp = torch.full((M,), 0.8, device=dev)
    top_k = torch.full((M,), 50, dtype=torch.int32, device=dev)
    top_p = torch.full((M,), 0.95, device=dev)
    u = torch.rand(M, device=dev, generator=torch.Generator(device=dev).manual_seed(1))
    ids = torch.empty(M, dtype=torch.int32, device=dev)

    ms_proj = timed(lambda: head.logits(x, rows, logits), args.steps, args.warmup)
    ms_samp = timed(lambda: HD.gllm_op_sample(logits, V, temp, top_k, top_p, u, ids), args.steps, args.warmup)
    ms_greedy = timed(lambda: HD.gllm_op_sample(logits, V, torch.zeros_like(temp), top_k, top_p, u, ids), args.steps, args.warmup)
    both = lambda: (head.logits(x, rows, logits), HD.gllm_op_sample(logits, V, temp, top_k, top_p, u, ids))
    ms_both = timed(both, args.steps, args.warmup)
    wbytes = V * H * 2
    result = {
        "metric": "rows given a next token per second (final norm + vocabulary projection + top-k/top-p sampling)",
        "value": round(M / (ms_both * 1e-3), 1), "unit": "rows/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_both, 4), "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"head hidden={H} vocab={V} rows={M}"},
        "roofline": {"kernel": "gemm_bf16_kernel (vocabulary projection)", "bound": "hbm",
                     "achieved": round(wbytes / (ms_proj * 1e-3) / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                     "frac": round(wbytes / (ms_proj * 1e-3) / 8e12, 4), "traffic": None,
                     "algorithmic_bytes": wbytes, "avg_launch_ms": round(ms_proj, 4),
                     "tflops": round(2.0 * M * V * H / (ms_proj * 1e-3) / 1e12, 1)},
        "sampler_ms": {"top_k_50_top_p_0.95": round(ms_samp, 4), "greedy": round(ms_greedy, 4)},
    }
    if not args.no_cpu_baseline:
        from oracle import head_oracle as Hd
        n = min(M, 4)
        xs = x[rows[:n].long()].cpu().numpy().astype(np.float64)
        gb, wb = synth.bf16_bits(gain.cpu()), synth.bf16_bits(w.cpu())
        lg = logits[:n, :V].cpu().numpy()
        t0 = time.perf_counter()
        ref = Hd.final_logits(xs, list(range(n)), gb, wb, 1e-6)
        toks = [Hd.sample(lg[i], 0.8, 50, 0.95, float(u[i])) for i in range(n)]
        secs = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": round(n / secs, 2), "unit": "rows/s", "cores": int(torch.get_num_threads()), "kind": "oracle",
                                  "sample": f"{n} rows of the same call, {secs:.1f} s"}
        err = float(np.abs(lg - ref).max())
        match = int(sum(int(ids[i]) == toks[i] for i in range(n)))
        result["check"] = {"logits_max_abs_vs_oracle": round(err, 5), "sampled_tokens_equal": f"{match}/{n}"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
