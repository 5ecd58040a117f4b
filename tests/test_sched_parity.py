"""The native scheduler (include/gllm_sched.h, through its ctypes binding) against the scheduling oracle:
integer work, so every comparison is exact -- budgets on a grid, micro-batch rows, block tables, finished
requests and counters step by step on random traces, and every field of the pipeline simulation."""
import os
import random
import re

import numpy as np
import pytest

from oracle import throttle_oracle as T
from paper_2504_14775_amd import binding as B
from paper_2504_14775_amd import sched as S

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "gllm_sched.h")


def both(**kw):
    base = dict(policy=T.THROTTLE, iters_t=8, max_p=2048, min_p=32, kv_thresh_bp=500, pp_depth=4, token_budget=2048,
                use_wt=True, use_ut=True, total_pages=4096)
    base.update(kw)
    return T.Params(**base), S.Params(**base)


def test_library_exports_every_function_the_header_declares():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    declared = sorted(set(re.findall(r"\b(gllm_sched_[a-z0-9_]+)\s*\(", text)))
    lib = B.load_host_library()
    for n in declared:
        assert hasattr(lib, n), n
    assert set(declared) == set(S.EXPORTS)


@pytest.mark.parametrize("kw", [dict(), dict(kv_thresh_bp=0), dict(use_wt=False), dict(use_ut=False),
                                dict(iters_t=3, max_p=512, min_p=1, kv_thresh_bp=2000, total_pages=777),
                                dict(use_wt=False, use_ut=False, pp_depth=7)])
def test_budgets_agree_on_a_grid(kw):
    po, pn = both(**kw)
    total = po.total_pages
    frees = sorted(set([0, 1, total // 20 - 1, total // 20, total // 20 + 1, total // 5, total // 2, total - 1, total]
                       + [random.Random(1).randrange(total + 1) for _ in range(5)]))
    for wp in [0, 1, 7, 31, 32, 33, 255, 256, 257, 4000, 16383, 16384, 16385, 10 ** 6, 10 ** 9]:
        for free in frees:
            assert S.gllm_sched_prefill_budget(pn, wp, free) == T.prefill_budget(po, wp, free), (wp, free)
    for rd in [0, 1, 3, 4, 5, 511, 512, 513, 10 ** 6]:
        assert S.gllm_sched_decode_budget(pn, rd) == T.decode_budget(po, rd)


def test_invalid_arguments_are_refused():
    _, pn = both()
    assert S.gllm_sched_prefill_budget(pn, -1, 10) == -1
    assert S.gllm_sched_prefill_budget(pn, 10, pn.total_pages + 1) == -1
    assert S.gllm_sched_decode_budget(pn, -5) == -1
    for bad in (dict(iters_t=0), dict(min_p=0), dict(max_p=16, min_p=32), dict(kv_thresh_bp=10000), dict(pp_depth=0),
                dict(policy=2), dict(total_pages=0), dict(token_budget=0)):
        with pytest.raises(B.GllmError) as e:
            S.Scheduler(both(**bad)[1])
        assert e.value.status == -1
    s = S.Scheduler(both(total_pages=10)[1])
    s.add_request(7, 20, 5)
    for args in ((7, 5, 5), (8, 0, 5), (8, 5, 0)):
        with pytest.raises(B.GllmError) as e:
            s.add_request(*args)
        assert e.value.status == -1
    with pytest.raises(B.GllmError) as e:
        s.add_request(9, 150, 20)                      # 170 tokens can never fit in 10 pages
    assert e.value.status == -2
    before = s.state()
    with pytest.raises(B.GllmError) as e:
        s.next_batch(capacity=0)
    assert e.value.status == -2 and s.state() == before
    with pytest.raises(B.GllmError):
        s.complete_batch(123)
    bid, rows = s.next_batch()
    assert rows == [(7, 20, 0)]
    with pytest.raises(B.GllmError) as e:
        s.block_tables(bid, 1, 1)                      # 2 pages do not fit a stride of 1
    assert e.value.status == -2
    assert s.block_tables(bid, 1, 4).tolist() == [[0, 1, -1, -1]]


@pytest.mark.parametrize("policy", [T.SARATHI, T.THROTTLE])
@pytest.mark.parametrize("pages,thresh,seed", [(4000, 500, 1), (260, 500, 2), (260, 0, 3), (150, 2500, 4)])
def test_step_by_step_agreement_on_random_traces(policy, pages, thresh, seed):
    po, pn = both(policy=policy, total_pages=pages, kv_thresh_bp=thresh, max_p=512, token_budget=512, pp_depth=3)
    so, sn = T.Scheduler(po), S.Scheduler(pn)
    rng = random.Random(seed)
    flying = []
    next_id = 0
    n_req = 90
    for step in range(20000):
        if next_id < n_req and rng.random() < 0.3:
            pl, ol = rng.randrange(1, 700), rng.randrange(1, 100)
            so.add_request(next_id, pl, ol)
            sn.add_request(next_id, pl, ol)
            next_id += 1
        if flying and (len(flying) >= po.pp_depth or rng.random() < 0.4):
            bid = flying.pop(rng.randrange(len(flying)) if rng.random() < 0.2 else 0)      # mostly in order
            assert sn.complete_batch(bid) == so.complete_batch(bid)
        go, gn = so.next_batch(), sn.next_batch()
        assert go == gn, step
        if go is not None:
            bid, rows = go
            flying.append(bid)
            stride = max(len(so.req[r].block_table) for r, _, _ in rows) + 1
            want = np.full((len(rows), stride), -1, dtype=np.int32)
            for i, (r, _, _) in enumerate(rows):
                want[i, :len(so.req[r].block_table)] = so.req[r].block_table
            assert np.array_equal(sn.block_tables(bid, len(rows), stride), want)
        st = sn.state()
        assert st["tokens_waiting"] == so.tokens_waiting() and st["decode_requests"] == so.n_decode
        assert st["free_pages"] == so.free_pages and st["batches_in_flight"] == len(so.in_flight)
        assert st["waiting_requests"] == len(so.waiting) and st["preemptions"] == so.preemptions
        if next_id == n_req and not flying and not so.waiting and not so.ready:
            break
    assert sorted(so.finished) == list(range(n_req))
    if pages <= 260 and (policy == T.SARATHI or thresh == 0):
        assert so.preemptions > 0            # small pools without head-room exercise the preemption rules


def arrivals_for(seed, n, mean_gap_ns, max_prompt, max_out):
    rng = random.Random(seed)
    t, out = 0, []
    for _ in range(n):
        t += int(rng.expovariate(1.0 / mean_gap_ns))
        out.append((t, rng.randrange(1, max_prompt), rng.randrange(1, max_out)))
    return out


@pytest.mark.parametrize("kw,seed", [
    (dict(policy=T.THROTTLE, total_pages=20000), 1), (dict(policy=T.SARATHI, total_pages=20000), 1),
    (dict(policy=T.THROTTLE, total_pages=1500, kv_thresh_bp=0), 2), (dict(policy=T.SARATHI, total_pages=1500), 2),
    (dict(policy=T.THROTTLE, use_wt=False, total_pages=6000), 3), (dict(policy=T.THROTTLE, use_ut=False, total_pages=6000), 3),
    (dict(policy=T.THROTTLE, pp_depth=1, iters_t=2, total_pages=6000), 4), (dict(policy=T.SARATHI, pp_depth=8, token_budget=512, total_pages=6000), 4),
])
def test_pipeline_simulation_agrees_field_by_field(kw, seed):
    po, pn = both(**kw)
    arrivals = arrivals_for(seed, 250, 40e6, 2500, 300)
    model = T.StageModel(base_ns=300_000, token_ns=33_000, decode_ctx_ns=13, prefill_pair_ns_per_1024=120)
    want = T.simulate(po, model, arrivals)
    got = S.gllm_sched_simulate(pn, (model.base_ns, model.token_ns, model.decode_ctx_ns, model.prefill_pair_ns_per_1024), arrivals)
    assert got == want


def test_simulation_rejects_bad_input():
    _, pn = both(total_pages=100)
    model = (1000, 10, 1, 1)
    with pytest.raises(B.GllmError) as e:
        S.gllm_sched_simulate(pn, model, [(5, 10, 10), (4, 10, 10)])          # arrivals must ascend
    assert e.value.status == -1
    with pytest.raises(B.GllmError) as e:
        S.gllm_sched_simulate(pn, model, [(0, 5000, 10)])                     # can never fit
    assert e.value.status == -2
