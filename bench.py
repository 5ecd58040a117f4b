#!/usr/bin/env python3
"""Benchmark of the stage forward on one MI355X: stage tokens/s on a mixed prefill+decode batch.

A step is one gllm_stage_forward over one batch: all layers of the stage, every kernel of the hot
path, inputs (weights, KV pool, hidden states) already resident in HBM; only the batch descriptor
(a few hundred KB of int32) crosses PCIe inside the call, as it does in serving.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config llama3_8b_pp4] [--no-cpu-baseline]

Eight untimed passes belong to the set-up (first-use costs), then W warm-up steps, then K timed steps between two
device synchronisations.  Prints ONE JSON line.  `roofline` describes the bf16 MFMA GEMM kernel (all four projections of a
layer are launches of it), measured with HIP events on the launch stream in a second pass of the
same steps; `roofline_decode_attention` gives the HBM figure of the decode attention kernel;
`cpu_baseline` times the CPU oracle on a bounded sample of the same batch.

    python bench.py --decode-rows 64 [--config llama3_8b_pp4]

runs a small decode-only micro-batch on the configuration's stage shape instead (not the headline workload): there
every kernel is a stream of weights or KV, and the line carries `roofline_whole_stage_streams`.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
SETUP_PASSES = 8            # untimed passes before the warm-up: first-use costs of every kernel and staging slot

# HBM-side bytes per launch come from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this very command (counters
# cannot be read from inside the process), scaled by a plain 1 GiB copy; their summaries are committed as
# profiles/stage_<config>_hbm_traffic.txt, each ending in a line
#   bench.py reads: gemm_bytes_per_launch=<float> decode_attention_bytes_per_launch=<float>
# A configuration without such a file reports traffic = null.
def measured_traffic(config):
    path = os.path.join(ROOT, "profiles", f"stage_{config}_hbm_traffic.txt")
    out = {"source": None}
    try:
        text = open(path).read()
    except OSError:
        return out
    import re
    for key in ("gemm", "decode_attention"):
        m = re.search(rf"{key}_bytes_per_launch=([0-9.eE+-]+)", text)
        if m:
            out[key] = float(m.group(1))
    out["source"] = f"profiles/stage_{config}_hbm_traffic.txt (offline rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of this command, copy-calibrated)"
    return out


def cpu_model():
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.startswith("model name"):
                return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def prefill_attn_flops(shape, batch):
    f = 0
    for n, c in zip(batch.new_tokens, batch.cached_len):
        n, c = int(n), int(c)
        if n > 1:
            f += 4 * shape.head_dim * shape.n_q_heads * (n * c + n * (n + 1) // 2)
    return f


def decode_kv_bytes(shape, batch):
    keys = sum(int(c) + 1 for n, c in zip(batch.new_tokens, batch.cached_len) if int(n) == 1)
    return keys * shape.kv_bytes_per_token_layer


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="llama3_8b_pp4")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--batch-index", type=int, default=0, help="batch of the 70B-shaped series")
    ap.add_argument("--layers", type=int, default=0, help="experiment: run only this many layers of the stage")
    ap.add_argument("--decode-rows", type=int, default=0, metavar="N",
                    help="instead of the configuration's batch: a decode-only micro-batch of N rows (contexts uniform in "
                         "1500..3500) on the configuration's stage shape -- the small-batch regime, bound by the weight "
                         "and KV streams; adds a whole-stage HBM roofline to the line")
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE",
                    help="experiment: gllm_stage_set_option(NAME, VALUE) before running")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile-pass", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run three plain 1 GiB device-to-device copies and exit (reference dispatches for "
                         "scaling the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU only (no sharding or collectives); "
                         "use --gpus 1.\n")
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2504_14775_amd import binding, synth
    if os.environ.get("GLLM_STAGE_LIBRARY"):      # another build of the library (experiments)
        binding.LIB_PATH = os.path.abspath(os.environ["GLLM_STAGE_LIBRARY"])

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible; the stage has no CPU path.\n")
        sys.exit(3)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": 1 << 30, "copies": 3}))
        return
    shape = synth.SHAPES[args.config]
    if args.layers > 0:
        import dataclasses
        shape = dataclasses.replace(shape, num_layers=args.layers)
    batch = (synth.make_decode_only_batch(args.decode_rows, args.seed) if args.decode_rows > 0
             else synth.make_batch(args.config, args.seed, args.batch_index))
    T = batch.num_tokens

    stage = binding.stage_for_batches(shape, [batch], device=dev)
    for opt in args.option:
        k, v = opt.split("=")
        stage.set_option(k, int(v))
    host_weights = []          # kept only if the oracle will be timed
    for l in range(shape.num_layers):
        w = synth.make_layer_weights(shape, args.seed, l, device=dev)
        stage.load_layer(l, w)
        if not args.no_cpu_baseline:
            host_weights.append({k: synth.bf16_bits(v) for k, v in w.items()})
        torch.cuda.synchronize()
        del w
    k_pool, v_pool = synth.make_pool(shape, args.seed, batch.num_blocks, device=dev)
    stage.bind_kv_pool(k_pool, v_pool, batch.num_blocks)
    hidden = synth.make_hidden(shape, args.seed, T, device=dev)
    out = torch.empty(T, shape.hidden, dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()

    # sample for the CPU baseline, taken before the forward touches the pool: more than 64 rows, so that the oracle's
    # many-rows loop nest is what is timed; if the stage is too deep for about 20 s of CPU work the oracle runs its
    # first layers only (stated in the output)
    sample = None
    cpu_layers = shape.num_layers
    if not args.no_cpu_baseline:
        dec = [i for i in range(batch.num_seqs) if batch.new_tokens[i] == 1][:24]
        pre = [i for i in range(batch.num_seqs) if batch.new_tokens[i] > 1][:1]
        ids = pre + dec
        nt = [min(int(batch.new_tokens[i]), 72 - len(dec)) for i in pre] + [1] * len(dec)
        if sum(nt) < 65:            # a decode-only batch: more decode rows
            dec = [i for i in range(batch.num_seqs) if batch.new_tokens[i] == 1][:72]
            ids, nt = pre + dec, nt[:len(pre)] + [1] * len(dec)
        sub, kp, vp, _ = synth.compact_subset(shape, batch, ids, nt, k_pool, v_pool)
        rows = []
        offs = batch.row_offsets
        for i, n in zip(ids, nt):
            rows += list(range(int(offs[i]), int(offs[i]) + n))
        sample = (sub, kp, vp, synth.bf16_bits(hidden[rows]))
        work_per_layer = sub.num_tokens * shape.gemm_flop_per_token_layer        # flop; the GEMMs dominate
        cpu_layers = max(1, min(shape.num_layers, int(6.0e11 // work_per_layer)))

    def step():
        stage.forward(batch.new_tokens, batch.cached_len, batch.block_tables, hidden, out)

    # first-use costs (code objects, every metadata staging slot, the clocks coming up from idle) are paid here, as
    # part of the set-up: with fewer than about eight passes before the timed region they add 10-20 ms to it
    for _ in range(SETUP_PASSES):
        step()
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    tokens_per_s = T * args.steps / elapsed

    # ---- per-kernel pass: HIP events on the launch stream around every kernel ----
    L = shape.num_layers
    gemm_flop_step = T * shape.gemm_flop_per_token_layer * L
    roofline = None
    extra = {}
    traffic = measured_traffic(args.config if args.decode_rows == 0 else "none")
    # operands once + result once, averaged over the four projections of a layer (result: fp32 planes for QKV, O and
    # down as planned for this row count, bf16 for gate/up)
    H_, I_, NQ, QD = shape.hidden, shape.intermediate, shape.n_qkv, shape.q_dim
    def _planes(n, k):
        return binding.gllm_op_gemm_plan(T, (n + 255) // 256 * 256, k, 0, 8)[1]
    alg_gemm_bytes = ((T * H_ * 2 + NQ * H_ * 2 + _planes(NQ, H_) * T * NQ * 4) + (T * QD * 2 + H_ * QD * 2 + _planes(H_, QD) * T * H_ * 4)
                      + (T * H_ * 2 + 2 * I_ * H_ * 2 + T * I_ * 2) + (T * I_ * 2 + H_ * I_ * 2 + _planes(H_, (I_ + 127) // 128 * 128) * T * H_ * 4)) / 4.0
    if not args.no_profile_pass:
        stage.set_profiling(True)
        for _ in range(args.steps):
            step()
        prof = stage.read_profile(reset=True)
        stage.set_profiling(False)
        per_step = {k: v[0] / args.steps for k, v in prof.items()}
        launches = {k: v[1] // args.steps for k, v in prof.items()}
        gemm_classes = ["gemm_qkv", "gemm_o", "gemm_gate_up_swiglu", "gemm_down"]
        gemm_ms = sum(per_step[c] for c in gemm_classes)
        gemm_launches = sum(launches[c] for c in gemm_classes)
        achieved = gemm_flop_step / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
        roofline = {"kernel": "gemm_bf16_kernel", "bound": "mfma", "achieved": round(achieved, 2),
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                    "traffic": traffic.get("gemm") if args.layers == 0 else None,
                    "traffic_unit": "bytes per launch (FETCH_SIZE + WRITE_SIZE, copy-calibrated; includes Infinity Cache hits)",
                    "traffic_source": traffic["source"],
                    "algorithmic_bytes_per_launch": alg_gemm_bytes,
                    "launches_per_step": gemm_launches,
                    "avg_launch_ms": round(gemm_ms / max(gemm_launches, 1), 5),
                    "flop_per_launch": gemm_flop_step / max(gemm_launches, 1)}
        H, I = shape.hidden, shape.intermediate
        per_class_flop = {"gemm_qkv": 2 * T * H * shape.n_qkv, "gemm_o": 2 * T * shape.q_dim * H,
                          "gemm_gate_up_swiglu": 4 * T * H * I, "gemm_down": 2 * T * H * I}
        extra["gemm_tflops_by_projection"] = {
            c: round(per_class_flop[c] * L / (per_step[c] * 1e-3) / 1e12, 1) for c in gemm_classes if per_step[c] > 0}
        kvb = decode_kv_bytes(shape, batch)
        if per_step.get("attn_decode", 0) > 0:
            gbs = kvb * L / (per_step["attn_decode"] * 1e-3) / 1e9
            extra["roofline_decode_attention"] = {
                "kernel": "decode_attention_kernel", "bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS,
                "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
                "traffic": traffic.get("decode_attention") if args.layers == 0 else None,
                "avg_launch_ms": round(per_step["attn_decode"] / L, 5), "bytes_per_launch": kvb}
        pf = prefill_attn_flops(shape, batch)
        if per_step.get("attn_prefill", 0) > 0:
            tf = pf * L / (per_step["attn_prefill"] * 1e-3) / 1e12
            extra["roofline_prefill_attention"] = {
                "kernel": "prefill_attention_kernel", "bound": "mfma", "achieved": round(tf, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / PEAK_BF16_TFLOPS, 4),
                "avg_launch_ms": round(per_step["attn_prefill"] / L, 5), "flop_per_launch": pf}
        if args.decode_rows > 0:
            # few rows: every kernel of the stage is a stream -- the weights once and the batch's KV once per layer
            stage_bytes = (shape.weight_elems_per_layer * 2 + kvb) * L
            gbs = stage_bytes / (ms_per_step * 1e-3) / 1e9
            extra["roofline_whole_stage_streams"] = {
                "bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(gbs / PEAK_HBM_GBS, 4), "bytes_per_step": stage_bytes,
                "note": "layer weights once + KV of the batch once, per layer, over the whole step time (all kernels)"}
        extra["kernel_ms_per_step"] = {k: round(v, 4) for k, v in per_step.items()}
        extra["kernel_ms_sum"] = round(sum(per_step.values()), 4)

    # ---- what this GPU sustains on a bare MFMA loop (bf16 operands like the GEMMs') and a bare streaming read ----
    sink = torch.randn(8192, device=dev).to(torch.bfloat16)
    probe = torch.empty(4 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    binding.gllm_op_peak_mfma(sink, 1024, 500); binding.gllm_op_peak_read(probe, probe.numel(), sink, 16384)
    binding.gllm_op_peak_read(probe, probe.numel(), sink, 16384, non_temporal=True)
    ev[0].record(); binding.gllm_op_peak_mfma(sink, 1024, 4000); ev[1].record()
    ev[2].record(); binding.gllm_op_peak_read(probe, probe.numel(), sink, 16384); ev[3].record()
    ev[4].record(); binding.gllm_op_peak_read(probe, probe.numel(), sink, 16384, non_temporal=True); ev[5].record()
    torch.cuda.synchronize()
    extra["ceiling_probes"] = {
        "mfma_loop_tflops": round(1024 * 4 * 4000 * 16 * 2 * 32 * 32 * 16 / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e12, 1),
        "stream_read_gbs": round(probe.numel() / (ev[2].elapsed_time(ev[3]) * 1e-3) / 1e9, 1),
        "stream_read_nontemporal_gbs": round(probe.numel() / (ev[4].elapsed_time(ev[5]) * 1e-3) / 1e9, 1),
        "note": "bare 32x32x16 bf16 MFMA loop on random operands / bare 16-byte streaming read of 4 GiB, plain and with "
                "the non-temporal hint, same box"}
    del probe

    # ---- CPU oracle on a bounded sample of the same batch ----
    cpu = None
    if sample is not None:
        import oracle
        sub, kp, vp, xs = sample
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        import dataclasses as _dc
        cpu_shape = _dc.replace(shape, num_layers=cpu_layers)
        per_layer = synth.pool_elems_per_layer(shape, sub.num_blocks)
        t0 = time.perf_counter()
        oracle.stage_forward(cpu_shape, host_weights[:cpu_layers], sub.new_tokens, sub.cached_len, sub.block_tables,
                             sub.num_blocks, kp[:cpu_layers * per_layer], vp[:cpu_layers * per_layer], xs)
        dt = time.perf_counter() - t0
        # tokens/s of the whole stage: rows per second through one layer, divided by the stage's layer count
        cpu = {"value": round(sub.num_tokens * cpu_layers / dt / L, 3), "unit": "tokens/s", "cores": cores, "kind": "oracle",
               "cpu_model": cpu_model(),
               "sample": f"{sub.num_tokens} token rows of the same batch ({int(sub.new_tokens[sub.new_tokens > 1].sum())} leading rows of a prefill "
                         f"chunk, {int((sub.new_tokens == 1).sum())} decode rows), {cpu_layers} of the {L} layers"
                         f"{'' if cpu_layers == L else ' (scaled to the whole stage)'}, {dt:.1f} s"}

    line = {
        "metric": "stage tokens/sec on mixed prefill+decode batch",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "setup_passes": SETUP_PASSES, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.config + (f"/decode_only_{args.decode_rows}" if args.decode_rows > 0 else "")
                               + (f"[first {args.layers} layers]" if args.layers > 0 else ""), "layers": L, "tokens_per_batch": T,
                   "prefill_tokens": int(batch.new_tokens[batch.new_tokens > 1].sum()),
                   "decode_seqs": int((batch.new_tokens == 1).sum()),
                   "mean_decode_context": float(np.mean(batch.cached_len[batch.new_tokens == 1])) if (batch.new_tokens == 1).any() else 0.0,
                   "seed": args.seed, "parallelism": "single GPU"},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    line.update(extra)
    print(json.dumps(line))
    stage.destroy()


if __name__ == "__main__":
    main()
