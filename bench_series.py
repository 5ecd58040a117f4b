#!/usr/bin/env python3
"""Per-batch latency of 16 consecutive hybrid batches on the 70B-shaped stage (20 layers of Llama-3-70B's shape on one
GPU, one shared KV pool), enqueued back to back on one stream with no host synchronisation in between: the
inter-batch imbalance the paper's scheduler exists to remove (section 2.4), seen from one stage.

    python bench_series.py [--passes R] [--seed S]

Prints one JSON line: per batch the prefill tokens P, decode rows D, keys read by the decode rows, (query, key) pairs
of prefill attention and the median stage time over R passes; and a least-squares fit of the linear stage-time model
that bench_sched.py's pipeline simulation uses (base + per new token + per decode key + per 1024 prefill pairs), with
its worst relative residual.
"""
import argparse
import json

import numpy as np
import torch

from paper_2504_14775_amd import binding, synth


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--passes", type=int, default=5)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    name = "llama3_70b_pp4"
    shape = synth.SHAPES[name]
    series = synth.make_series(name, args.seed)
    stage = binding.stage_for_batches(shape, series, device=dev)
    for l in range(shape.num_layers):
        w = synth.make_layer_weights(shape, args.seed, l, device=dev)
        stage.load_layer(l, w)
        torch.cuda.synchronize()
        del w
    nb = series[0].num_blocks
    k_pool, v_pool = synth.make_pool(shape, args.seed, nb, device=dev)
    stage.bind_kv_pool(k_pool, v_pool, nb)
    hidden = [synth.make_hidden(shape, args.seed + 100 + i, b.num_tokens, device=dev) for i, b in enumerate(series)]
    outs = [torch.empty(b.num_tokens, shape.hidden, dtype=torch.bfloat16, device=dev) for b in series]
    torch.cuda.synchronize()

    times = []
    for p in range(args.passes + 1):                       # the first pass warms up
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(series) + 1)]
        ev[0].record()
        for i, b in enumerate(series):
            stage.forward(b.new_tokens, b.cached_len, b.block_tables, hidden[i], outs[i])
            ev[i + 1].record()
        torch.cuda.synchronize()
        if p > 0:
            times.append([ev[i].elapsed_time(ev[i + 1]) for i in range(len(series))])
    ms = np.median(np.asarray(times), axis=0)

    rows, feats = [], []
    for i, b in enumerate(series):
        nt, cl = b.new_tokens.astype(np.int64), b.cached_len.astype(np.int64)
        dec, pre = nt == 1, nt > 1
        keys = int((cl[dec] + 1).sum())
        pairs = int((nt[pre] * cl[pre] + nt[pre] * (nt[pre] + 1) // 2).sum())
        rows.append({"batch": i, "tokens": int(nt.sum()), "prefill_tokens": int(nt[pre].sum()), "decode_rows": int(dec.sum()),
                     "decode_keys": keys, "prefill_pairs": pairs, "ms": round(float(ms[i]), 3)})
        feats.append([1.0, float(nt.sum()), float(keys), pairs / 1024.0])
    A, y = np.asarray(feats), ms * 1e6                      # ns
    coef, *_ = np.linalg.lstsq(A, y, rcond=None)
    resid = np.abs(A @ coef - y) / y
    total_tokens = sum(r["tokens"] for r in rows)
    print(json.dumps({
        "metric": "stage time per batch, 16 consecutive hybrid batches back to back", "unit": "ms", "data": "synthetic",
        "config": {"workload": name, "layers": shape.num_layers, "passes": args.passes, "seed": args.seed},
        "series_ms": round(float(ms.sum()), 2), "tokens_per_s": round(total_tokens / (float(ms.sum()) * 1e-3), 1),
        "min_ms": round(float(ms.min()), 3), "max_ms": round(float(ms.max()), 3), "batches": rows,
        "stage_time_model_ns": {"base": round(float(coef[0])), "per_token": round(float(coef[1]), 1),
                                "per_decode_key": round(float(coef[2]), 2), "per_1024_prefill_pairs": round(float(coef[3]), 1),
                                "worst_relative_residual": round(float(resid.max()), 4)},
    }))


if __name__ == "__main__":
    main()
