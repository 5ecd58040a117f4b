"""A closed generation loop on the GPU: scheduler -> embedding -> stage -> final norm + projection -> sampler -> the
sampled tokens go back into the requests (section 2.1 and 3 of the paper put together, one pipeline stage holding
the whole tiny model).

The oracles follow with teacher forcing: they are fed the token ids the GPU actually used, keep their own KV pool,
and must agree on every micro-batch -- embedding bit-exact, hidden states and logits within the stage's tolerance,
and every greedy token must be (within that tolerance) a maximiser of the oracle's logits.  The run includes
chunked prompts, decode rows, several micro-batches in flight and, in the small-pool case, preemption with
recomputation of a request whose generated tokens have become part of its prompt.
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from oracle import head_oracle as Hd
from paper_2504_14775_amd import head as HD
from paper_2504_14775_amd import sched as S
from paper_2504_14775_amd import synth
from gpu_util import DEV, GpuStage, bits_of, to_dev_bits
from helpers import layer_weights_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("pages,expect_preemption", [(64, False), (7, True)])
def test_generation_loop_with_teacher_forced_oracles(pages, expect_preemption):
    print(f"generation loop, pool of {pages} pages", flush=True)
    shape = dataclasses.replace(synth.SHAPES["tiny"], num_layers=2, name="tiny_lm")
    V, H = 300, shape.hidden
    rng = np.random.default_rng(5)
    prompts = [rng.integers(0, V, size=n).tolist() for n in (37, 5, 70, 16, 1, 23)]
    out_len = [6, 9, 4, 7, 10, 3]
    table = synth.bf16_bits(synth.normal_bf16(31, 1, 0, V * H, 1.0, 0.0)).reshape(V, H)
    gain = synth.bf16_bits(synth.normal_bf16(31, 2, 0, H, 0.1, 1.0))
    w_lm = synth.bf16_bits(synth.normal_bf16(31, 3, 0, V * H, 0.02, 0.0)).reshape(V, H)
    w = layer_weights_np(shape, 31)

    params = S.Params(policy=S.TOKEN_THROTTLING, iters_t=2, max_p=48, min_p=4, kv_thresh_bp=0 if expect_preemption else 500,
                      pp_depth=2, token_budget=40, total_pages=pages)
    sch = S.Scheduler(params)
    sizing = synth.Batch(np.array([48] * 2 + [1] * 4, dtype=np.int32), np.array([100] * 6, dtype=np.int32),
                         np.zeros((6, 12), dtype=np.int32), pages)
    stage = GpuStage(shape, w, [sizing])
    head = HD.Head(H, V, 8, shape.rms_eps)
    d_table, d_wlm = to_dev_bits(table), to_dev_bits(w_lm)
    head.load(to_dev_bits(gain), d_wlm)
    n_el = shape.num_layers * synth.pool_elems_per_layer(shape, pages)
    blank = np.full(n_el, 0x7FC1, dtype=np.uint16)
    kp, vp = blank.copy(), blank.copy()
    dk, dv = to_dev_bits(blank), to_dev_bits(blank)

    tokens = [list(p) for p in prompts]                   # everything known of a request: prompt, then generated tokens
    for r, (p, o) in enumerate(zip(prompts, out_len)):
        sch.add_request(r, len(p), o)
    flying, finished, produced, worst_h, worst_l = [], [], [0] * len(prompts), 0.0, 0.0
    for _ in range(500):
        got = sch.next_batch()
        if got is not None:
            bid, rows = got
            nt = np.array([n for _, n, _ in rows], dtype=np.int32)
            cl = np.array([c for _, _, c in rows], dtype=np.int32)
            bt = sch.block_tables(bid, len(rows), 12)
            ids = np.concatenate([np.asarray(tokens[r][c:c + n], dtype=np.int32) for r, n, c in rows])
            assert len(ids) == int(nt.sum())
            ends = np.cumsum(nt) - 1
            takers = [i for i, (r, n, c) in enumerate(rows) if c + n == len(tokens[r])]      # rows that yield a token
            # ---- GPU: embedding -> stage -> head -> greedy ----
            x = torch.empty(len(ids), H, dtype=torch.bfloat16, device=DEV)
            HD.gllm_op_embedding(torch.from_numpy(ids).to(DEV), d_table, x)
            out, out32 = stage.run(synth.Batch(nt, cl, bt, pages), dk, dv, x)
            sel = torch.from_numpy(ends[takers].astype(np.int32)).to(DEV)
            logits = torch.empty(len(takers), head.padded_vocab, dtype=torch.float32, device=DEV)
            picked = torch.empty(len(takers), dtype=torch.int32, device=DEV)
            if takers:
                head.logits(out32, sel, logits)
                zeros = torch.zeros(len(takers), device=DEV)
                HD.gllm_op_sample(logits, V, zeros, torch.zeros(len(takers), dtype=torch.int32, device=DEV), zeros + 1, zeros, picked)
            torch.cuda.synchronize()
            # ---- oracles on the same ids ----
            xe = Hd.embedding(table, ids)
            assert np.array_equal(bits_of(x), xe)
            ref, _ = oracle.stage_forward(shape, w, nt, cl, bt, pages, kp, vp, xe)
            rms = float(np.sqrt((ref ** 2).mean()))
            err_h = float(np.abs(out32.cpu().numpy() - ref).max()) / max(1.0, rms)
            assert err_h <= 2e-2
            worst_h = max(worst_h, err_h)
            if takers:
                want = Hd.final_logits(ref, ends[takers], gain, w_lm, shape.rms_eps)
                got_l = logits[:, :V].cpu().numpy().astype(np.float64)
                err_l = float(np.abs(got_l - want).max())
                assert err_l <= 2e-2
                worst_l = max(worst_l, err_l)
                pk = picked.cpu().numpy()
                for j, i in enumerate(takers):
                    assert pk[j] == int(np.argmax(got_l[j]))                     # greedy on the GPU's own logits: exact
                    assert want[j, pk[j]] >= want[j].max() - 2 * err_l - 1e-12   # and a maximiser of the oracle's, within tolerance
                    tokens[rows[i][0]].append(int(pk[j]))
                    produced[rows[i][0]] += 1
            flying.append(bid)
        if flying and (got is None or len(flying) == params.pp_depth):
            finished += sch.complete_batch(flying.pop(0))
        if len(finished) == len(prompts):
            break
    assert sorted(finished) == list(range(len(prompts))) and not flying
    st = sch.state()
    assert st["free_pages"] == pages
    assert (st["preemptions"] > 0) == expect_preemption
    for r in range(len(prompts)):
        assert len(tokens[r]) == len(prompts[r]) + out_len[r]                    # exactly the requested number of new tokens kept
        assert produced[r] >= out_len[r]                                         # (recomputation re-derives some)
    print(f"[generate] hidden err {worst_h:.3g} (scaled), logits err {worst_l:.3g}, {st['preemptions']} preemptions", flush=True)
    head.destroy()
