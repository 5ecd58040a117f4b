"""The scheduler drives the stage library: a small serving loop on the GPU.

Requests go through the native Token Throttling scheduler (include/gllm_sched.h); every micro-batch it forms
(new-token counts, cached lengths, block tables from its page allocator) is handed unchanged to
gllm_stage_forward() and, independently, to the CPU oracle of the stage, each side keeping its own KV pool
across the whole run.  This checks what neither component's own tests can: that the descriptors the scheduler
emits are valid stage inputs (pages in range, no page shared between requests, chunk boundaries and decode
positions consistent with what is in the cache), also across preemption and recomputation.
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2504_14775_amd import sched as S
from paper_2504_14775_amd import synth
from gpu_util import GpuStage, bits_of, parity_report, to_dev_bits
from helpers import hidden_np, layer_weights_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("policy,pages,thresh", [(S.TOKEN_THROTTLING, 64, 500), (S.CHUNKED_PREFILL, 64, 500),
                                                 (S.TOKEN_THROTTLING, 7, 0), (S.CHUNKED_PREFILL, 12, 0)])
def test_scheduler_batches_run_on_the_stage_and_match_the_oracle(policy, pages, thresh):
    print(f"serving loop policy={policy} pages={pages} thresh={thresh}", flush=True)
    shape = dataclasses.replace(synth.SHAPES["tiny"], name="tiny_serve")
    prompts = [37, 5, 70, 16, 1, 23, 48]
    outputs = [4, 6, 3, 5, 8, 2, 7]
    params = S.Params(policy=policy, iters_t=2, max_p=48, min_p=4, kv_thresh_bp=thresh, pp_depth=2, token_budget=40,
                      total_pages=pages)
    sch = S.Scheduler(params)
    w = layer_weights_np(shape, 21)
    # one hidden-state row per (request, position): what the previous stage would hand over for that token
    span = max(p + o for p, o in zip(prompts, outputs)) + sum(outputs)       # room for recomputed prompts
    rows_of = [hidden_np(shape, 100 + r, span) for r in range(len(prompts))]
    n_el = shape.num_layers * synth.pool_elems_per_layer(shape, pages)
    blank = np.full(n_el, 0x7FC1, dtype=np.uint16)                            # NaN pattern: unwritten slots must never leak
    kp, vp = blank.copy(), blank.copy()
    dk, dv = to_dev_bits(blank), to_dev_bits(blank)
    sizing = synth.Batch(np.array([48] * 2 + [1] * 5, dtype=np.int32), np.array([100] * 7, dtype=np.int32),
                         np.zeros((7, 12), dtype=np.int32), pages)
    stage = GpuStage(shape, w, [sizing])
    for r, (p, o) in enumerate(zip(prompts, outputs)):
        sch.add_request(r, p, o)
    flying, finished, n_batches, worst = [], [], 0, 0.0
    for _ in range(400):
        got = sch.next_batch()
        if got is not None:
            bid, rows = got
            n_batches += 1
            nt = np.array([n for _, n, _ in rows], dtype=np.int32)
            cl = np.array([c for _, _, c in rows], dtype=np.int32)
            bt = sch.block_tables(bid, len(rows), 12)
            x = np.concatenate([rows_of[r][c:c + n] for r, n, c in rows])
            batch = synth.Batch(nt, cl, bt, pages)
            ref, _ = oracle.stage_forward(shape, w, nt, cl, bt, pages, kp, vp, x)
            out, out32 = stage.run(batch, dk, dv, to_dev_bits(x))
            rep = parity_report(f"batch {bid} ({len(rows)} rows, {int(nt.sum())} tokens)", bits_of(out), out32.cpu().numpy(), ref)
            assert np.array_equal(bits_of(out), bits_of(out32.to(torch.bfloat16)))
            assert rep["max_abs_f32_scaled"] <= 2e-2 and rep["mean_rel_bf16"] <= 5e-3
            worst = max(worst, rep["max_abs_f32_scaled"])
            flying.append(bid)
        if flying and (got is None or len(flying) == params.pp_depth):
            finished += sch.complete_batch(flying.pop(0))
        if len(finished) == len(prompts):
            break
    assert sorted(finished) == list(range(len(prompts))) and not flying
    st = sch.state()
    assert st["free_pages"] == pages and st["tokens_waiting"] == 0 and st["decode_requests"] == 0
    # both pools were written at exactly the same places (the oracle's pool is the placement reference)
    gk, gv = bits_of(dk), bits_of(dv)
    assert np.array_equal(gk == 0x7FC1, kp == 0x7FC1) and np.array_equal(gv == 0x7FC1, vp == 0x7FC1)
    if pages < 64:
        assert st["preemptions"] > 0         # the tiny pools force recomputation, and parity held through it
    print(f"[serve] {n_batches} micro-batches, {st['preemptions']} preemptions, worst scaled error {worst:.3g}", flush=True)
