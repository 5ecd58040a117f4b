"""The serving loop of paper_2504_14775_amd/engine.py on the GPU: several micro-batches enqueued ahead of their
completion, sampled tokens fed back, against the oracles with teacher forcing (the oracles are fed the token ids the
engine used and keep their own KV pool): embedding bit-exact, hidden states and logits within the stage's tolerance,
every greedy token a maximiser of the oracle's logits within that tolerance; sampled tokens (temperature > 0) must be
tokens the oracle's kept set contains.  Cases: a roomy pool, a pool small enough to preempt, prefix caching."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from oracle import head_oracle as Hd
from paper_2504_14775_amd import engine as E
from paper_2504_14775_amd import sched as S
from paper_2504_14775_amd import synth
from gpu_util import DEV, bits_of, to_dev_bits
from helpers import layer_weights_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("pages,depth,caching,sampled,lanes", [(64, 3, False, False, 1), (7, 2, False, False, 1), (64, 2, True, False, 1),
                                                               (64, 2, False, True, 1), (64, 4, False, False, 2), (7, 2, True, False, 2)])
def test_engine_generates_what_the_oracles_confirm(pages, depth, caching, sampled, lanes):
    print(f"engine: pool of {pages} pages, depth {depth}, prefix caching {caching}, sampling {sampled}, {lanes} lane(s)", flush=True)
    shape = dataclasses.replace(synth.SHAPES["tiny"], num_layers=2, name="tiny_engine")
    V, H = 300, shape.hidden
    rng = np.random.default_rng(9)
    stem = rng.integers(0, V, size=40).tolist()
    prompts = [stem + rng.integers(0, V, size=n).tolist() for n in (9, 30)] + \
              [rng.integers(0, V, size=n).tolist() for n in (37, 5, 1, 23)]
    out_len = [6, 9, 4, 7, 10, 3]
    table = synth.bf16_bits(synth.normal_bf16(51, 1, 0, V * H, 1.0, 0.0)).reshape(V, H)
    gain = synth.bf16_bits(synth.normal_bf16(51, 2, 0, H, 0.1, 1.0))
    w_lm = synth.bf16_bits(synth.normal_bf16(51, 3, 0, V * H, 0.02, 0.0)).reshape(V, H)
    w = layer_weights_np(shape, 51)
    params = S.Params(policy=S.TOKEN_THROTTLING, iters_t=2, max_p=48, min_p=4, kv_thresh_bp=0 if pages < 64 else 500,
                      pp_depth=depth, token_budget=40, total_pages=pages, prefix_caching=caching)
    eng = E.Engine(shape, V, params, max_batch_tokens=64, max_batch_seqs=8, max_context=192, lanes=lanes)
    d_table = to_dev_bits(table)
    eng.load([{k: to_dev_bits(v) for k, v in lw.items()} for lw in w], d_table, to_dev_bits(gain), to_dev_bits(w_lm))
    n_el = shape.num_layers * synth.pool_elems_per_layer(shape, pages)
    kp, vp = np.zeros(n_el, dtype=np.uint16), np.zeros(n_el, dtype=np.uint16)
    worst = {"h": 0.0, "l": 0.0, "batches": 0, "max_flying": 0}

    def check(slot):
        """Called when a micro-batch is retired, oldest first -- the order in which the GPU ran them."""
        worst["batches"] += 1
        worst["max_flying"] = max(worst["max_flying"], len(eng.flying) + 1)
        rows, T = slot.rows, slot.num_tokens
        nt = np.array([n for _, n, _ in rows], dtype=np.int32)
        cl = np.array([c for _, _, c in rows], dtype=np.int32)
        bt = eng.sched.block_tables(slot.batch_id, len(rows), eng.max_blocks)
        ids = slot.ids_host.numpy()[:T].copy()
        xe = Hd.embedding(table, ids)
        assert np.array_equal(bits_of(slot.x[:T]), xe)
        ref, _ = oracle.stage_forward(shape, w, nt, cl, bt, pages, kp, vp, xe)
        rms = float(np.sqrt((ref ** 2).mean()))
        err_h = float(np.abs(slot.out32[:T].cpu().numpy() - ref).max()) / max(1.0, rms)
        assert err_h <= 2e-2
        worst["h"] = max(worst["h"], err_h)
        m = len(slot.takers)
        if m == 0:
            return
        ends = np.cumsum(nt) - 1
        want = Hd.final_logits(ref, ends[slot.takers], gain, w_lm, shape.rms_eps)
        got_l = slot.logits[:m, :V].cpu().numpy().astype(np.float64)
        err_l = float(np.abs(got_l - want).max())
        assert err_l <= 2e-2
        worst["l"] = max(worst["l"], err_l)
        pk = slot.picked_host.numpy()[:m]
        for j, i in enumerate(slot.takers):
            sp = eng.requests[rows[i][0]].sampling
            if sp.temperature <= 0:
                assert pk[j] == int(np.argmax(got_l[j]))
                assert want[j, pk[j]] >= want[j].max() - 2 * err_l - 1e-12
            else:
                keep, _ = Hd.kept_distribution(got_l[j], sp.temperature, sp.top_k, sp.top_p)
                assert keep[pk[j]], (j, pk[j])

    eng.observer = check
    late = [1] if caching else []                          # the second prompt with the stem arrives when the first is cached
    for r, (p, o) in enumerate(zip(prompts, out_len)):
        sp = E.Sampling(temperature=0.8, top_k=20, top_p=0.9, seed=r) if sampled else None
        if r not in late:
            eng.add_request(r, p, o, sp)
    result = eng.run()
    for r in late:
        eng.add_request(r, prompts[r], out_len[r])
        result = eng.run()
    if caching and pages >= 64:
        # a follow-up that repeats a finished conversation: the pages of the answer are found as well
        before = eng.sched.state()["prefix_hit_tokens"]
        talk = prompts[1] + result[1]                       # 70 prompt tokens + 9 answer tokens
        prompts.append(talk + rng.integers(0, V, size=12).tolist())
        out_len.append(3)
        eng.add_request(6, prompts[6], out_len[6])
        result = eng.run()
        assert len(talk) == 79 and eng.sched.state()["prefix_hit_tokens"] - before == 64   # 4 whole pages of the 78 cached positions
    st = eng.sched.state()
    assert {r: len(t) for r, t in result.items()} == dict(enumerate(out_len))
    assert st["free_pages"] == pages and st["batches_in_flight"] == 0
    assert worst["max_flying"] == depth                     # micro-batches really were enqueued ahead
    if pages < 64 and not caching:
        assert st["preemptions"] > 0
    if caching and pages >= 64:
        assert st["prefix_hit_tokens"] >= 32                # the second prompt found the first one's stem
    for r, toks in result.items():
        assert all(0 <= t < V for t in toks)
    print(f"[engine] {worst['batches']} micro-batches, hidden err {worst['h']:.3g}, logits err {worst['l']:.3g}, "
          f"{st['preemptions']} preemptions, {st['prefix_hit_tokens']} prefix-hit tokens", flush=True)
    eng.close()


def test_streams_picked_for_the_lanes_are_distinct_and_usable():
    print("stream calibration", flush=True)
    cur = torch.cuda.current_stream()
    for n, beside in ((0, ()), (1, (cur,)), (3, ())):
        got = E.independent_streams(n, DEV, beside=beside)
        assert len(got) == n and len({s.cuda_stream for s in got}) == n
        assert all(s.cuda_stream != cur.cuda_stream for s in got)
        x = torch.zeros(8, device=DEV)
        for s in got:
            with torch.cuda.stream(s):
                x += 1                                      # (serialised below: one stream at a time)
            s.synchronize()
        assert float(x[0]) == n
