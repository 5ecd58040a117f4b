#!/usr/bin/env python3
"""Closed-loop generation on one GPU: requests -> scheduler -> embedding -> stage -> final norm + vocabulary projection
-> sampler -> tokens back into the requests (paper_2504_14775_amd/engine.py), with the 8 layers of the Llama-3-8B-shaped
stage standing for the whole model (hidden 4096, vocabulary 128256, random weights).

    python bench_engine.py [--requests N] [--seed S]

Prints one JSON line.  `value` = generated tokens per second (wall clock, everything included: scheduling, block
tables, token-id upload, the kernels, the read-back of the sampled ids) in the engine's default arrangement (`two_lanes`):
up to #PP_depth micro-batches enqueued ahead, consecutive micro-batches on two streams through two stage objects over
one set of weights, the last-stage extras of each on a further stream.  `enqueued_ahead` runs all layers on one stream
(extras still beside them); `enqueued_ahead_one_stream` keeps the extras on that stream too; `synchronous` also keeps only
one micro-batch in flight, i.e. exposes the host work; `gpu_busy` is the sum of the micro-batches' own event-timed
durations over the wall time (above 1 when they overlap).  --try-lanes N... times further lane counts.
All requests are present at the start;
prompt and output lengths are log-normal (medians 220 and 64), a stand-in for a chat workload.
`serving` replays the same requests with Poisson arrivals at --rate requests per second (wall clock) and reports the
latency metrics of the paper's section 4.1: time to first token, time per output token, end-to-end latency.
"""
import argparse
import json
import math
import random
import time

import torch

from paper_2504_14775_amd import engine as E
from paper_2504_14775_amd import sched as S
from paper_2504_14775_amd import synth


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--requests", type=int, default=1024)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--try-lanes", type=int, nargs="*", default=[], help="experiment: further lane counts to time")
    ap.add_argument("--rate", type=float, default=100.0, help="arrivals per second of the serving run (0: skip it)")
    args = ap.parse_args()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    shape = synth.SHAPES["llama3_8b_pp4"]
    V, H = 128256, shape.hidden
    rng = random.Random(args.seed)
    reqs = []
    for _ in range(args.requests):
        p = int(min(2048, max(4, rng.lognormvariate(math.log(220), 0.9))))
        o = int(min(256, max(1, rng.lognormvariate(math.log(64), 0.6))))
        reqs.append(([rng.randrange(V) for _ in range(p)], o))
    layers = [synth.make_layer_weights(shape, args.seed, l, device=dev) for l in range(shape.num_layers)]
    table = synth.normal_bf16(args.seed, 901, 0, V * H, 1.0, 0.0, device=dev).view(V, H)
    gain = synth.normal_bf16(args.seed, 902, 0, H, 0.1, 1.0, device=dev)
    w_vocab = synth.normal_bf16(args.seed, 903, 0, V * H, 0.02, 0.0, device=dev).view(V, H)
    params = S.Params(policy=S.TOKEN_THROTTLING, iters_t=8, max_p=2048, min_p=32, kv_thresh_bp=500, pp_depth=4,
                      token_budget=2048, total_pages=32768)

    def run(max_in_flight, overlap_head=True, lanes=2):
        eng = E.Engine(shape, V, params, max_batch_tokens=2048 + args.requests, max_batch_seqs=args.requests + 8,
                       max_context=2048 + 256, device=dev, max_in_flight=max_in_flight, timing=True, overlap_head=overlap_head,
                       lanes=lanes)
        eng.load(layers, table, gain, w_vocab)
        for i, (p, o) in enumerate(reqs):
            eng.add_request(i, p, o, E.Sampling(temperature=0.8, top_k=50, top_p=0.95, seed=i))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out = eng.run()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        st = dict(eng.stats)
        assert all(len(out[i]) == reqs[i][1] for i in range(len(reqs)))
        eng.close()
        return {"generated_tokens_per_s": round(st["tokens_generated"] / wall, 1),
                "computed_tokens_per_s": round(st["tokens_computed"] / wall, 1), "wall_s": round(wall, 3),
                "micro_batches": st["micro_batches"], "mean_tokens_per_micro_batch": round(st["tokens_computed"] / st["micro_batches"], 1),
                "ms_per_micro_batch": round(wall * 1e3 / st["micro_batches"], 3), "gpu_busy": round(st["gpu_ms"] * 1e-3 / wall, 4)}

    def serve(rate):
        """Poisson arrivals on the wall clock; a request is admitted when its time has come."""
        eng = E.Engine(shape, V, params, max_batch_tokens=2048 + args.requests, max_batch_seqs=args.requests + 8,
                       max_context=2048 + 256, device=dev)
        eng.load(layers, table, gain, w_vocab)
        arr, t = [], 0.0
        for _ in reqs:
            t += rng.expovariate(rate)
            arr.append(t)
        first, last, nxt, done = {}, {}, 0, 0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        while done < len(reqs):
            now = time.perf_counter() - t0
            while nxt < len(reqs) and arr[nxt] <= now:
                eng.add_request(nxt, reqs[nxt][0], reqs[nxt][1], E.Sampling(temperature=0.8, top_k=50, top_p=0.95, seed=nxt))
                nxt += 1
            news = eng.step()
            now = time.perf_counter() - t0
            for rid, _, ended in news:
                first.setdefault(rid, now)
                if ended:
                    last[rid] = now
                    done += 1
            if not news and not eng.flying and nxt < len(reqs):
                time.sleep(max(0.0, min(arr[nxt] - (time.perf_counter() - t0), 0.002)))
        wall = time.perf_counter() - t0
        eng.close()
        ttft = sorted(first[i] - arr[i] for i in range(len(reqs)))
        e2e = sorted(last[i] - arr[i] for i in range(len(reqs)))
        tpot = sorted((last[i] - first[i]) / (reqs[i][1] - 1) for i in range(len(reqs)) if reqs[i][1] > 1)
        pct = lambda v, q: round(1e3 * v[min(len(v) - 1, int(q * len(v)))], 2)
        return {"arrival_rate_per_s": rate, "wall_s": round(wall, 2), "generated_tokens_per_s": round(sum(o for _, o in reqs) / wall, 1),
                "ttft_ms": {"mean": round(1e3 * sum(ttft) / len(ttft), 2), "p50": pct(ttft, 0.5), "p99": pct(ttft, 0.99)},
                "tpot_ms": {"mean": round(1e3 * sum(tpot) / len(tpot), 2), "p50": pct(tpot, 0.5), "p99": pct(tpot, 0.99)},
                "e2e_ms": {"mean": round(1e3 * sum(e2e) / len(e2e), 2), "p50": pct(e2e, 0.5), "p99": pct(e2e, 0.99)}}

    run(None)                                               # warm-up: first-use costs of every kernel
    two_lanes = run(None)
    ahead = run(None, lanes=1)
    more = {n: run(None, lanes=n) for n in args.try_lanes}
    one_stream = run(None, overlap_head=False, lanes=1)
    sync = run(1, overlap_head=False, lanes=1)
    print(json.dumps({
        "metric": "generated tokens per second, closed loop on one GPU (scheduler + embedding + stage + head + sampler)",
        "value": two_lanes["generated_tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "higher_is_better": True, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.requests} requests at once, 8 layers of the Llama-3-8B shape as the whole model, vocabulary {V}",
                   "prompt_tokens": sum(len(p) for p, _ in reqs), "output_tokens": sum(o for _, o in reqs),
                   "scheduler": "token throttling T=8 MaxP=2048 MinP=32 KV_thresh=0.05 depth=4", "sampling": "temperature 0.8, top-k 50, top-p 0.95"},
        "two_lanes": two_lanes, "enqueued_ahead": ahead, **{f"lanes_{n}": v for n, v in more.items()}, "enqueued_ahead_one_stream": one_stream, "synchronous": sync, "serving": serve(args.rate) if args.rate > 0 else None}))


if __name__ == "__main__":
    main()
