"""The native KV page pool (include/gllm_kv.h) and the native scheduler with prefix caching against their oracles:
integer work, so every comparison is exact -- page ids, holders, registration flags, eviction counts after every
operation of random traffic, micro-batch rows and block tables step by step, every field of the simulation."""
import os
import random
import re

import numpy as np
import pytest

from oracle import kv_oracle as K
from oracle import throttle_oracle as T
from paper_2504_14775_amd import binding as B
from paper_2504_14775_amd import kv as KV
from paper_2504_14775_amd import sched as S

PAGE = 16
HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "gllm_kv.h")


def test_library_exports_every_function_the_header_declares():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    declared = sorted(set(re.findall(r"\b(gllm_kv_[a-z0-9_]+)\s*\(", text)))
    lib = B.load_host_library()
    for n in declared:
        assert hasattr(lib, n), n
    assert set(declared) == set(KV.EXPORTS)


def same_state(po, pn):
    st = pn.state()
    assert st["free_pages"] == len(po.free) and st["idle_cached_pages"] == len(po.queue)
    assert st["registered_pages"] == len(po.index) and st["evictions"] == po.evictions
    assert pn.available() == po.available()
    for page in range(po.total):
        assert pn.page_info(page) == (po.count[page], po.key[page] is not None, po.children[page]), page


@pytest.mark.parametrize("seed,total", [(0, 5), (1, 16), (2, 64), (3, 300)])
def test_pool_operations_agree_on_random_traffic(seed, total):
    rng = random.Random(seed)
    po, pn = K.PagePool(total), KV.PagePool(total)
    stems = [[rng.randrange(4) for _ in range(PAGE * 6)] for _ in range(4)]
    held = []
    for step in range(2500):
        if held and (rng.random() < 0.45 or po.available() == 0):
            tokens, pages = held.pop(rng.randrange(len(held)))
            po.release(pages)
            pn.release(pages)
        else:
            stem = rng.choice(stems)
            tokens = stem[:rng.randrange(0, len(stem) + 1)] + [rng.randrange(4, 60) for _ in range(rng.randrange(1, 50))]
            bound = (len(tokens) - 1) // PAGE
            pages = po.match(tokens, bound)
            assert pn.match(tokens, bound) == pages
            want = -(-len(tokens) // PAGE)
            registering = True
            while len(pages) < want and po.available() > 0:
                p = po.alloc()
                assert pn.alloc() == [p]
                i = len(pages)
                pages.append(p)
                if registering and (i + 1) * PAGE <= len(tokens):
                    parent = pages[i - 1] if i else K.ROOT
                    ok = po.register(parent, tokens[i * PAGE:(i + 1) * PAGE], p)
                    assert pn.register(parent, tokens[i * PAGE:(i + 1) * PAGE], p) == ok
                    registering = ok
            held.append((tokens, pages))
        if step % 25 == 0 or total <= 16:
            same_state(po, pn)
    for tokens, pages in held:
        po.release(pages)
        pn.release(pages)
    same_state(po, pn)
    assert pn.available() == total


def test_allocating_several_pages_at_once_takes_them_in_single_page_order():
    po, pn = K.PagePool(10), KV.PagePool(10)
    assert pn.alloc(4) == [po.alloc() for _ in range(4)] == [0, 1, 2, 3]
    assert pn.alloc(0) == []
    pn.release([2, 0])
    po.release([2, 0])
    assert pn.alloc(3) == [po.alloc() for _ in range(3)] == [0, 2, 4]


def test_invalid_calls_are_refused_and_change_nothing():
    for bad in (0, -3, 2 ** 31):
        with pytest.raises(B.GllmError) as e:
            KV.PagePool(bad)
        assert e.value.status == -1
    pn = KV.PagePool(4)
    a, b = pn.alloc(2)
    before = pn.state()
    with pytest.raises(B.GllmError) as e:
        pn.alloc(3)                                        # only 2 left
    assert e.value.status == -2 and pn.state() == before
    ones = [1] * PAGE
    for parent, page in ((K.ROOT, 3), (K.ROOT, 4), (K.ROOT, -1), (b, a), (a, a), (7, a)):
        with pytest.raises(B.GllmError) as e:              # page not held / out of range / parent not registered
            pn.register(parent, ones, page)
        assert e.value.status == -1
    assert pn.register(K.ROOT, ones, a)
    with pytest.raises(B.GllmError):
        pn.register(K.ROOT, [2] * PAGE, a)                 # already registered
    for pages in ([a, a], [3], [9], [-1], [a, b, 2]):
        with pytest.raises(B.GllmError) as e:
            pn.release(pages)
        assert e.value.status == -1
    assert pn.page_info(a) == (1, True, 0) and pn.page_info(b) == (1, False, 0)
    pn.release([a, b])
    assert pn.state() == dict(total_pages=4, free_pages=3, idle_cached_pages=1, registered_pages=1, evictions=0)
    assert pn.available() == 4
    with pytest.raises(B.GllmError):
        pn.page_info(4)


# ---- the scheduler with prefix caching ------------------------------------------------------------------------

def both(**kw):
    base = dict(policy=T.THROTTLE, iters_t=8, max_p=512, min_p=32, kv_thresh_bp=500, pp_depth=3, token_budget=512,
                use_wt=True, use_ut=True, total_pages=4096, prefix_caching=True)
    base.update(kw)
    return T.Params(**base), S.Params(**base)


def shared_prompt(rng, stems, max_tail):
    stem = rng.choice(stems)
    return stem[:rng.randrange(0, len(stem) + 1)] + [rng.randrange(10, 30000) for _ in range(rng.randrange(1, max_tail))]


@pytest.mark.parametrize("report", [False, True])
@pytest.mark.parametrize("policy", [T.SARATHI, T.THROTTLE])
@pytest.mark.parametrize("pages,thresh,seed", [(4000, 500, 1), (260, 500, 2), (260, 0, 3), (120, 1000, 4)])
def test_step_by_step_agreement_with_shared_prefixes(policy, pages, thresh, seed, report):
    po, pn = both(policy=policy, total_pages=pages, kv_thresh_bp=thresh)
    so, sn = T.Scheduler(po), S.Scheduler(pn)
    rng = random.Random(seed)
    stems = [[rng.randrange(10) for _ in range(rng.randrange(100, 600))] for _ in range(5)]
    flying, next_id, n_req = [], 0, 90
    rows_of = {}
    history = []                                     # finished conversations: a later request may continue one
    text = {}
    for step in range(20000):
        if next_id < n_req and rng.random() < 0.3:
            prompt, ol = shared_prompt(rng, stems, 200), rng.randrange(1, 100)
            if report and history and rng.random() < 0.3:
                prompt = rng.choice(history) + [rng.randrange(10, 30000) for _ in range(rng.randrange(1, 60))]
                prompt = prompt[:700]
            text[next_id] = list(prompt)
            if rng.random() < 0.15:
                so.add_request(next_id, len(prompt), ol)                 # some requests come without content
                sn.add_request(next_id, len(prompt), ol)
            else:
                so.add_request(next_id, len(prompt), ol, prompt)
                sn.add_request(next_id, len(prompt), ol, prompt)
            next_id += 1
        if flying and (len(flying) >= po.pp_depth or rng.random() < 0.4):
            bid = flying.pop(rng.randrange(len(flying)) if rng.random() < 0.2 else 0)
            toks = None
            if report:                               # a made-up token per row; some are withheld
                toks = [(-1 if rng.random() < 0.02 else (r * 7919 + c + n) % 30000) for r, n, c in rows_of[bid]]
                for (r, n, c), t in zip(rows_of[bid], toks):
                    q = so.req[r]
                    if q.tokens is not None and t >= 0 and c + n == len(text[r]) and c + n >= q.prompt_len:
                        text[r].append(t)            # the conversation as a client would see it
            ended = so.complete_batch(bid, toks)
            assert sn.complete_batch(bid, toks) == ended
            history += [text[r] for r in ended if so.req[r].tokens is not None]
        go, gn = so.next_batch(), sn.next_batch()
        assert go == gn, step
        if go is not None:
            bid, rows = go
            flying.append(bid)
            rows_of[bid] = rows
            stride = max(len(so.req[r].block_table) for r, _, _ in rows) + 1
            want = np.full((len(rows), stride), -1, dtype=np.int32)
            for i, (r, _, _) in enumerate(rows):
                want[i, :len(so.req[r].block_table)] = so.req[r].block_table
            assert np.array_equal(sn.block_tables(bid, len(rows), stride), want)
        st = sn.state()
        assert st["tokens_waiting"] == so.tokens_waiting() and st["decode_requests"] == so.n_decode
        assert st["free_pages"] == so.free_pages and st["idle_cached_pages"] == len(so.pool.queue)
        assert st["prefix_hit_tokens"] == so.hit_tokens and st["evictions"] == so.pool.evictions
        assert st["preemptions"] == so.preemptions and st["waiting_requests"] == len(so.waiting)
        if next_id == n_req and not flying and not so.waiting and not so.ready:
            break
    assert sorted(so.finished) == list(range(n_req))
    assert so.hit_tokens > 0
    if pages <= 260:
        assert so.pool.evictions > 0


def test_without_the_switch_token_ids_are_ignored():
    po, pn = both(prefix_caching=False, total_pages=64, pp_depth=1, iters_t=1)
    so, sn = T.Scheduler(po), S.Scheduler(pn)
    a = list(range(64))
    for sch in (so, sn):
        sch.add_request(0, 64, 1, a)
        bid, rows = sch.next_batch()
        sch.complete_batch(bid)
        sch.add_request(1, 64, 1, a)
        assert sch.next_batch()[1] == [(1, 64, 0)]
    assert sn.state()["prefix_hit_tokens"] == 0 and sn.state()["idle_cached_pages"] == 0


def arrivals_with_content(seed, n, mean_gap_ns, n_stems, stem_len, max_tail, max_out):
    rng = random.Random(seed)
    stems = [[rng.randrange(1000) for _ in range(stem_len)] for _ in range(n_stems)]
    t, out = 0, []
    for _ in range(n):
        t += int(rng.expovariate(1.0 / mean_gap_ns))
        prompt = rng.choice(stems) + [rng.randrange(1000, 30000) for _ in range(rng.randrange(1, max_tail))]
        out.append((t, len(prompt), rng.randrange(1, max_out), prompt))
    return out


@pytest.mark.parametrize("kw,seed", [
    (dict(policy=T.THROTTLE, total_pages=20000), 1), (dict(policy=T.SARATHI, total_pages=20000), 1),
    (dict(policy=T.THROTTLE, total_pages=1500, kv_thresh_bp=0), 2), (dict(policy=T.SARATHI, total_pages=1500), 2),
    (dict(policy=T.THROTTLE, total_pages=6000, prefix_caching=False), 3),
])
def test_pipeline_simulation_with_content_agrees_field_by_field(kw, seed):
    po, pn = both(max_p=2048, token_budget=2048, pp_depth=4, **kw)
    arrivals = arrivals_with_content(seed, 200, 40e6, 4, 1500, 1000, 300)
    model = T.StageModel(base_ns=300_000, token_ns=33_000, decode_ctx_ns=13, prefill_pair_ns_per_1024=120)
    want = T.simulate(po, model, arrivals)
    got = S.gllm_sched_simulate(pn, (model.base_ns, model.token_ns, model.decode_ctx_ns, model.prefill_pair_ns_per_1024), arrivals)
    assert got == want
    assert (want["prefix_hit_tokens"] > 0) == kw.get("prefix_caching", True)
