"""Prefix caching end to end on the GPU: the native scheduler with its page pool (include/gllm_kv.h) hands block
tables whose leading pages are shared between requests to gllm_stage_forward().

Two references.  (1) The stage oracle is fed the same descriptors and keeps its own pool: every micro-batch must
agree within the stage's tolerance, and both pools must have been written at the same places.  (2) What caching
must not change: for every request the oracle also runs the whole prompt alone, uncached, in a private pool; the
row that yields the request's first token must equal that run's last row -- bit for bit inside the oracle (its
rows do not depend on how a prompt is cut or on who computed the prefix), within tolerance on the GPU.
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2504_14775_amd import sched as S
from paper_2504_14775_amd import synth
from gpu_util import GpuStage, bits_of, parity_report, to_dev_bits
from helpers import layer_weights_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("pages,expect", [(64, {0: 0, 1: 48, 2: 64, 3: 0, 4: 32}), (5, None)])
def test_shared_prefix_pages_give_the_same_rows_as_uncached_prompts(pages, expect):
    print(f"prefix caching, pool of {pages} pages", flush=True)
    shape = dataclasses.replace(synth.SHAPES["tiny"], num_layers=2, name="tiny_prefix")
    V, H = 200, shape.hidden
    rng = np.random.default_rng(11)
    stem = rng.integers(0, V, size=52).tolist()
    prompts = [stem + rng.integers(0, V, size=18).tolist(),           # 70 tokens: 4 whole pages
               stem + rng.integers(0, V, size=9).tolist(),            # shares 3 whole pages with the first
               None,                                                  # the first prompt again
               rng.integers(0, V, size=30).tolist(),                  # nothing shared
               stem[:32] + rng.integers(0, V, size=13).tolist()]      # shares 2 whole pages
    prompts[2] = list(prompts[0])
    out_len = [3, 2, 2, 2, 4]
    table = synth.bf16_bits(synth.normal_bf16(41, 1, 0, V * H, 1.0, 0.0)).reshape(V, H)
    w = layer_weights_np(shape, 41)
    params = S.Params(policy=S.TOKEN_THROTTLING, iters_t=2, max_p=48, min_p=4, kv_thresh_bp=0, pp_depth=2, token_budget=40,
                      total_pages=pages, prefix_caching=True)
    sch = S.Scheduler(params)
    sizing = synth.Batch(np.array([48] * 2 + [1] * 4, dtype=np.int32), np.array([100] * 6, dtype=np.int32),
                         np.zeros((6, 12), dtype=np.int32), pages)
    stage = GpuStage(shape, w, [sizing])
    n_el = shape.num_layers * synth.pool_elems_per_layer(shape, pages)
    blank = np.full(n_el, 0x7FC1, dtype=np.uint16)
    kp, vp = blank.copy(), blank.copy()
    dk, dv = to_dev_bits(blank), to_dev_bits(blank)

    # generated tokens are made up (no head in this test): request r's j-th output token is a fixed function of r, j
    tokens = [list(p) + [(7 * r + 3 * j) % V for j in range(o)] for r, (p, o) in enumerate(zip(prompts, out_len))]
    first_cached, first_row_gpu, first_row_ref = {}, {}, {}
    sch.add_request(0, len(prompts[0]), out_len[0], prompts[0])
    added = 1
    flying, finished = [], []
    for _ in range(400):
        got = sch.next_batch()
        if got is not None:
            bid, rows = got
            nt = np.array([n for _, n, _ in rows], dtype=np.int32)
            cl = np.array([c for _, _, c in rows], dtype=np.int32)
            bt = sch.block_tables(bid, len(rows), 12)
            ids = np.concatenate([np.asarray(tokens[r][c:c + n], dtype=np.int64) for r, n, c in rows])
            x = table[ids]
            ref, _ = oracle.stage_forward(shape, w, nt, cl, bt, pages, kp, vp, x)
            out, out32 = stage.run(synth.Batch(nt, cl, bt, pages), dk, dv, to_dev_bits(x))
            rep = parity_report(f"batch {bid} rows={[(r, int(n), int(c)) for r, n, c in rows]}", bits_of(out), out32.cpu().numpy(), ref)
            assert rep["max_abs_f32_scaled"] <= 2e-2 and rep["mean_rel_bf16"] <= 5e-3
            ends = np.cumsum(nt) - 1
            got32 = out32.cpu().numpy()
            for i, (r, n, c) in enumerate(rows):
                if c < len(prompts[r]) and r not in first_cached:
                    first_cached[r] = c                                  # cached length of the request's first chunk
                if c + n == len(prompts[r]):                             # the row that yields the first output token
                    first_row_gpu[r], first_row_ref[r] = got32[ends[i]], ref[ends[i]]
            flying.append(bid)
        if flying and (got is None or len(flying) == params.pp_depth):
            finished += sch.complete_batch(flying.pop(0))
        if added == 1 and sch.state()["decode_requests"] >= 1:             # the first prompt is in the cache: add the others
            for r in range(1, len(prompts)):
                sch.add_request(r, len(prompts[r]), out_len[r], prompts[r])
            added = len(prompts)
        if len(finished) == len(prompts):
            break
    assert sorted(finished) == list(range(len(prompts))) and not flying
    st = sch.state()
    assert st["free_pages"] == pages and st["prefix_hit_tokens"] > 0
    if expect is not None:
        assert first_cached == expect and st["prefix_hit_tokens"] == sum(expect.values()) and st["preemptions"] == 0
    else:
        assert st["evictions"] > 0                                          # the small pool recycles cached pages
    gk, gv = bits_of(dk), bits_of(dv)
    assert np.array_equal(gk == 0x7FC1, kp == 0x7FC1) and np.array_equal(gv == 0x7FC1, vp == 0x7FC1)
    # (2) every prompt alone, uncached, in a private pool
    worst = 0.0
    for r, p in enumerate(prompts):
        n_pages = -(-len(p) // 16)
        n_priv = shape.num_layers * synth.pool_elems_per_layer(shape, n_pages)
        pk, pv = np.full(n_priv, 0x7FC1, dtype=np.uint16), np.full(n_priv, 0x7FC1, dtype=np.uint16)
        alone, _ = oracle.stage_forward(shape, w, np.array([len(p)], dtype=np.int32), np.array([0], dtype=np.int32),
                                        np.arange(n_pages, dtype=np.int32)[None, :], n_pages, pk, pv, table[np.asarray(p)])
        assert np.array_equal(first_row_ref[r], alone[-1]), r              # caching is exact inside the oracle
        rms = float(np.sqrt((alone ** 2).mean()))
        err = float(np.abs(first_row_gpu[r] - alone[-1]).max()) / max(1.0, rms)
        assert err <= 2e-2, (r, err)
        worst = max(worst, err)
    print(f"[prefix] first chunks started at {first_cached}, {st['prefix_hit_tokens']} tokens skipped, {st['evictions']} evictions, "
          f"{st['preemptions']} preemptions, worst error against uncached prompts {worst:.3g}", flush=True)
