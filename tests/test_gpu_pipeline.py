"""Two pipeline stages on one GPU: two stage objects, each with half of the layers and its own KV pool, sharing one
set of page tables (section 3.3 of the paper), micro-batches from the scheduler handed from the first to the second
through device memory.  What one GPU can show of pipelining: with two micro-batches in flight (stage 0 of batch j+1
on one stream while stage 1 of batch j runs on another, ordered by events only) every output is bit-identical to
running the batches one stage after the other with a device synchronisation in between, and both agree with the
stage oracle applied twice (bf16 activations between the stages, as between two workers).
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2504_14775_amd import sched as S
from paper_2504_14775_amd import synth
from gpu_util import DEV, GpuStage, bits_of, to_dev_bits
from helpers import hidden_np, layer_weights_np

pytestmark = pytest.mark.gpu


def test_two_stages_with_two_micro_batches_in_flight():
    print("two stages on two streams", flush=True)
    whole = dataclasses.replace(synth.SHAPES["tiny"], num_layers=4, name="tiny_pp2")
    half = dataclasses.replace(whole, num_layers=2, name="tiny_pp2_stage")
    pages = 48
    w = layer_weights_np(whole, 61)
    prompts, outputs = [37, 5, 70, 16, 1, 23, 48], [4, 6, 3, 5, 8, 2, 7]
    params = S.Params(policy=S.TOKEN_THROTTLING, iters_t=2, max_p=48, min_p=4, kv_thresh_bp=500, pp_depth=2, token_budget=40,
                      total_pages=pages)
    sch = S.Scheduler(params)
    for r, (p, o) in enumerate(zip(prompts, outputs)):
        sch.add_request(r, p, o)
    span = max(p + o for p, o in zip(prompts, outputs))
    rows_of = [hidden_np(whole, 300 + r, span) for r in range(len(prompts))]
    # the schedule is fixed first (it does not depend on activations), then replayed three ways
    batches, flying, finished = [], [], []
    for _ in range(400):
        got = sch.next_batch()
        if got is not None:
            bid, rows = got
            nt = np.array([n for _, n, _ in rows], dtype=np.int32)
            cl = np.array([c for _, _, c in rows], dtype=np.int32)
            x = np.concatenate([rows_of[r][c:c + n] for r, n, c in rows])
            batches.append((synth.Batch(nt, cl, sch.block_tables(bid, len(rows), 12), pages), x))
            flying.append(bid)
        if flying and (got is None or len(flying) == params.pp_depth):
            finished += sch.complete_batch(flying.pop(0))
        if len(finished) == len(prompts):
            break
    assert len(finished) == len(prompts) and len(batches) >= 10
    sizing = synth.Batch(np.array([48] * 2 + [1] * 5, dtype=np.int32), np.array([100] * 7, dtype=np.int32),
                         np.zeros((7, 12), dtype=np.int32), pages)
    stages = [GpuStage(half, w[:2], [sizing]), GpuStage(half, w[2:], [sizing])]
    n_el = half.num_layers * synth.pool_elems_per_layer(half, pages)
    blank = np.full(n_el, 0x7FC1, dtype=np.uint16)

    def run(pipelined):
        pools = [(to_dev_bits(blank), to_dev_bits(blank)) for _ in range(2)]
        for st, (k, v) in zip(stages, pools):
            st.stage.bind_kv_pool(k, v, pages)
        streams = [torch.cuda.Stream(), torch.cuda.Stream()] if pipelined else [torch.cuda.current_stream()] * 2
        outs = []
        torch.cuda.synchronize()
        for b, x in batches:
            T = b.num_tokens
            xin = to_dev_bits(x)
            mid = torch.empty(T, half.hidden, dtype=torch.bfloat16, device=DEV)
            out = torch.empty(T, half.hidden, dtype=torch.bfloat16, device=DEV)
            handoff = torch.cuda.Event()
            if pipelined:
                streams[0].wait_stream(torch.cuda.current_stream())      # the inputs were made on the current stream
                streams[1].wait_stream(torch.cuda.current_stream())
            stages[0].stage.forward(b.new_tokens, b.cached_len, b.block_tables, xin, mid, None, stream=streams[0])
            handoff.record(streams[0])
            streams[1].wait_event(handoff)
            stages[1].stage.forward(b.new_tokens, b.cached_len, b.block_tables, mid, out, None, stream=streams[1])
            if not pipelined:
                torch.cuda.synchronize()
            outs.append((xin, mid, out))                                 # kept alive until the final synchronisation
        torch.cuda.synchronize()
        return [bits_of(o) for _, _, o in outs], [bits_of(k) for k, _ in pools]

    seq_out, seq_pools = run(False)
    pipe_out, pipe_pools = run(True)
    for j, (a, b) in enumerate(zip(seq_out, pipe_out)):
        assert np.array_equal(a, b), j
    for a, b in zip(seq_pools, pipe_pools):
        assert np.array_equal(a, b)
    # the oracle, stage after stage, bf16 between the stages
    pools = [(blank.copy(), blank.copy()), (blank.copy(), blank.copy())]
    worst = 0.0
    for j, (b, x) in enumerate(batches):
        _, mid16 = oracle.stage_forward(half, w[:2], b.new_tokens, b.cached_len, b.block_tables, pages, pools[0][0], pools[0][1], x)
        ref, _ = oracle.stage_forward(half, w[2:], b.new_tokens, b.cached_len, b.block_tables, pages, pools[1][0], pools[1][1], mid16)
        got = oracle.bf16_to_f64(pipe_out[j])
        rms = float(np.sqrt((ref ** 2).mean()))
        err = float(np.abs(got - ref).max()) / max(1.0, rms)
        rel = float(np.abs(got - ref).sum() / np.abs(ref).sum())
        assert err <= 2e-2 + 2.0 ** -8 * float(np.abs(ref).max()) / max(1.0, rms) and rel <= 5e-3, (j, err, rel)
        worst = max(worst, rel)
    print(f"[pipeline] {len(batches)} micro-batches, two in flight: bit-identical to the synchronised run; worst mean rel error "
          f"against the two-stage oracle {worst:.3g}", flush=True)
