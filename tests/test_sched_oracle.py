"""Pins of the scheduling oracle (oracle/throttle_oracle.py) against what the paper fixes: the values of
Eq. 1, Eq. 2, Eq. 3 and Eq. 4 worked by hand for the paper's hyper-parameters (section 4.1: #T = 8,
#MaxP = 2048, #MinP = 32, KV_thresh = 0.05), the special cases in which Eq. 3 must reduce to Eq. 1 or Eq. 2,
the behaviour the two case studies describe in words (sections 3.1 and 3.2), and conservation laws that any
correct scheduler obeys (every request produces exactly its output length, pages are never shared and all come
back)."""
import random

import pytest

from oracle import throttle_oracle as T


def paper_params(**kw):
    return T.Params(**{**dict(policy=T.THROTTLE, iters_t=8, max_p=2048, min_p=32, kv_thresh_bp=500, pp_depth=4,
                              token_budget=2048, total_pages=10000), **kw})


# ---- Eq. 1 .. Eq. 4, numbers worked by hand -------------------------------------------------------------------
@pytest.mark.parametrize("wp,want", [(16384, 2048), (100000, 2048), (8000, 1000), (8001, 1001), (300, 38), (256, 32),
                                     (100, 32), (33, 32), (20, 20), (1, 1), (0, 0)])
def test_eq1_waiting_tokens_throttle(wp, want):
    """Eq. 1: #P = min(max(#WP / #T, #MinP), #MaxP) with an empty cache; never more than what waits."""
    p = paper_params(kv_thresh_bp=0)
    assert T.prefill_budget(p, wp, p.total_pages) == want


@pytest.mark.parametrize("free,want", [(10000, 2048), (5000, 1024), (2500, 512), (157, 32), (156, 32), (100, 32), (0, 32)])
def test_eq2_idle_rate_throttle(free, want):
    """Eq. 2: #P = max(#MaxP x KV_free, #MinP), with so many tokens waiting that Eq. 1's term is at its cap."""
    p = paper_params(kv_thresh_bp=0)
    assert T.prefill_budget(p, 10 ** 6, free) == want      # 2048 * 0.0157 = 32.15 -> 32; below that #MinP holds


@pytest.mark.parametrize("free,want", [(10000, 2048), (5000, 970), (1000, 107), (600, 32), (500, 32), (499, 0), (0, 0)])
def test_eq3_with_threshold(free, want):
    """Eq. 3 idle-rate term: 2048 x (KV_free - 0.05) / 0.95: 0.5 -> 970.1, 0.1 -> 107.8, 0.06 -> 21.6 (-> #MinP);
    an idle rate below the threshold suspends prefill."""
    p = paper_params()
    assert T.prefill_budget(p, 10 ** 6, free) == want


def test_eq3_takes_the_smaller_of_its_two_terms():
    p = paper_params()
    assert T.prefill_budget(p, 4000, 5000) == 500          # waiting term 4000/8 = 500 < idle term 970
    assert T.prefill_budget(p, 16000, 5000) == 970         # idle term 970 < waiting term 2000
    assert T.prefill_budget(p, 4000, 600) == 32            # both small: #MinP
    assert T.prefill_budget(p, 4000, 499) == 0


def test_ablations_drop_one_term_each():
    assert T.prefill_budget(paper_params(use_wt=False), 4000, 5000) == 970
    assert T.prefill_budget(paper_params(use_ut=False), 4000, 5000) == 500
    assert T.prefill_budget(paper_params(use_ut=False), 10 ** 6, 600) == 2048
    assert T.prefill_budget(paper_params(use_ut=False), 10 ** 6, 499) == 0       # the threshold still suspends
    assert T.prefill_budget(paper_params(use_wt=False, use_ut=False), 5000, 5000) == 2048


def test_eq3_is_monotone_and_bounded():
    p = paper_params()
    rng = random.Random(3)
    for _ in range(300):
        wp, free = rng.randrange(1, 40000), rng.randrange(0, p.total_pages + 1)
        v = T.prefill_budget(p, wp, free)
        assert 0 <= v <= min(wp, p.max_p)
        if free * 10000 >= p.kv_thresh_bp * p.total_pages:
            assert v >= min(wp, p.min_p)
        assert T.prefill_budget(p, wp + rng.randrange(1, 500), free) >= v
        assert T.prefill_budget(p, wp, min(p.total_pages, free + rng.randrange(1, 500))) >= v


@pytest.mark.parametrize("rd,depth,want", [(0, 4, 0), (1, 4, 1), (4, 4, 1), (5, 4, 2), (512, 4, 128), (513, 4, 129), (10, 3, 4)])
def test_eq4_decode_budget(rd, depth, want):
    assert T.decode_budget(paper_params(pp_depth=depth), rd) == want


# ---- the case studies ---------------------------------------------------------------------------------------
def drain_prefill(policy, iters_t, arrivals_tokens, steps):
    """Requests with one output token each arrive at once; returns the prefill tokens of consecutive micro-batches
    (each completed before the next is formed, as with a pipeline of depth 1)."""
    s = T.Scheduler(paper_params(policy=policy, iters_t=iters_t, pp_depth=1, min_p=1, total_pages=100000))
    for i, n in enumerate(arrivals_tokens):
        s.add_request(i, n, 1)
    out = []
    for _ in range(steps):
        got = s.next_batch()
        if got is None:
            out.append(0)
            continue
        out.append(sum(n for _, n, _ in got[1]))
        s.complete_batch(got[0])
    return out


def test_case_study_prefill_spread_over_iterations():
    """Section 3.2, first scenario (#T = 3, nothing waiting before): the baseline takes the whole arrival in
    its first micro-batch and has no prefill tokens in the next; throttling hands out a third of what waits,
    each time, so the following micro-batches all carry prefill work."""
    base = drain_prefill(T.SARATHI, 3, [600, 600, 600], 4)
    ours = drain_prefill(T.THROTTLE, 3, [600, 600, 600], 4)
    assert base == [1800, 0, 0, 0]
    assert ours == [600, 400, 267, 178]          # ceil(1800/3), ceil(1200/3), ceil(800/3), ceil(533/3)


def test_case_study_prefill_follows_cache_pressure():
    """Section 3.2, second scenario: plenty of tokens waiting.  The baseline takes its full budget without looking
    at the cache, runs the pool empty, is left with micro-batches that carry decode rows only and has to preempt;
    throttling shrinks its prefill share as the cache fills, keeps the threshold's head-room and preempts nobody."""
    def run(policy):
        s = T.Scheduler(paper_params(policy=policy, pp_depth=1, total_pages=1000))
        for i in range(40):
            s.add_request(i, 1000, 400)
        shares, frees = [], []
        for _ in range(30):
            got = s.next_batch()
            shares.append(sum(n for _, n, c in got[1] if not (n == 1 and c >= 1000)))
            frees.append(s.free_pages)
            s.complete_batch(got[0])
        return shares, frees, s.preemptions
    base, base_free, base_preempted = run(T.SARATHI)
    ours, ours_free, ours_preempted = run(T.THROTTLE)
    assert base[0] == 2048 and base[1] == 2046              # budget minus the decode rows, whatever the cache holds
    assert min(base_free) == 0 and 0 in base and base_preempted > 0
    assert ours[0] == 2048 and ours == sorted(ours, reverse=True) and min(ours) == 32
    assert ours[1] == 2048 * (8710 - 500) // 9500           # Eq. 3 with 871 of 1000 pages free
    assert min(ours_free) >= 50 and ours_preempted == 0


def test_case_study_decode_rows_are_spread_over_the_pipeline():
    """Section 3.3 (pipeline depth 4): with #RD requests decoding, throttling puts ceil(#RD / 4) rows in each
    micro-batch, so the four micro-batches in flight cover every request once; the baseline puts all of them in
    the first micro-batch and leaves the next three empty."""
    def run(policy):
        s = T.Scheduler(paper_params(policy=policy, total_pages=100000))
        for i in range(10):
            s.add_request(i, 20, 50)
        while True:                                           # prefill everything, one micro-batch at a time
            got = s.next_batch()
            if got is None or all(n == 1 and c >= 20 for _, n, c in got[1]):
                break
            s.complete_batch(got[0])
        sizes, seen = [len(got[1])], [r for r, _, _ in got[1]]
        for _ in range(3):
            got = s.next_batch()
            sizes.append(0 if got is None else len(got[1]))
            seen += [] if got is None else [r for r, _, _ in got[1]]
        return sizes, seen
    ours, seen = run(T.THROTTLE)
    assert ours == [3, 3, 3, 1] and sorted(seen) == list(range(10))
    base, _ = run(T.SARATHI)
    assert base == [10, 0, 0, 0]


# ---- conservation laws on random traces ----------------------------------------------------------------------
@pytest.mark.parametrize("policy", [T.SARATHI, T.THROTTLE])
@pytest.mark.parametrize("pages,thresh", [(4000, 500), (300, 500), (300, 0)])
def test_every_request_completes_and_pages_are_conserved(policy, pages, thresh):
    rng = random.Random(pages + thresh + policy)
    s = T.Scheduler(paper_params(policy=policy, total_pages=pages, kv_thresh_bp=thresh, max_p=512, token_budget=512))
    want = {}
    flying = []
    produced = {}
    next_id = 0
    for step in range(6000):
        if next_id < 120 and rng.random() < 0.3:
            pl, ol = rng.randrange(1, 900), rng.randrange(1, 120)
            s.add_request(next_id, pl, ol)
            want[next_id] = ol
            produced[next_id] = 0
            next_id += 1
        if flying and (len(flying) >= s.p.pp_depth or rng.random() < 0.4):
            bid, rows = flying.pop(0)
            for rid, n, c in rows:
                r = s.req[rid]
                if n == 1 and c == r.prompt_len + r.generated - 1 and r.prefilled >= r.prompt_len:
                    produced[rid] += 1                                   # a decode row yields one token
                elif c + n == r.prompt_len:
                    produced[rid] += 1                                   # the chunk that completes the prompt too
            s.complete_batch(bid)
        got = s.next_batch()
        if got is not None:
            flying.append(got)
            assert len(flying) <= s.p.pp_depth
            ids = [r for r, _, _ in got[1]]
            assert len(set(ids)) == len(ids)
            for rid, n, c in got[1]:
                assert n >= 1 and c >= 0 and len(s.req[rid].block_table) == T.ceil_div(c + n, T.PAGE)
        owned = [pg for r in s.req.values() for pg in r.block_table]
        assert len(owned) == len(set(owned)) and len(owned) + s.free_pages == pages
        assert sum(len(rows) for _, rows in flying) == sum(r.in_flight for r in s.req.values())
        if next_id == 120 and not flying and not s.waiting and not s.ready:
            break
    assert next_id == 120 and sorted(s.finished) == list(range(120)) and s.free_pages == pages
    # a preempted request recomputes, but the tokens it hands to the user are counted once: output_len in total
    for rid, ol in want.items():
        assert produced[rid] >= ol
        assert s.req[rid].generated == s.req[rid].output_len
    if pages == 4000:
        assert s.preemptions == 0 and all(produced[r] == want[r] for r in want)


def test_a_zero_threshold_preempts_more():
    """Section 4.4 (sensitivity to KV_thresh): with no head-room the cache runs full and running requests have to
    be preempted and recomputed; the threshold keeps room for the decode rows."""
    rng = random.Random(9)
    t, arrivals = 0, []
    for _ in range(150):
        t += rng.randrange(1, 30_000_000)
        arrivals.append((t, rng.randrange(100, 1500), rng.randrange(50, 400)))
    res = {th: T.simulate(paper_params(total_pages=1200, kv_thresh_bp=th), T.StageModel(), arrivals) for th in (0, 500, 2000)}
    assert res[0]["preemptions"] > res[500]["preemptions"] >= res[2000]["preemptions"]


def test_simulated_pipeline_shows_the_papers_effect():
    """Not a number from the paper, only its direction (section 4.2): under the same arrivals token throttling
    leaves fewer bubbles in the last stage and a smaller spread of micro-batch sizes than the baseline."""
    rng = random.Random(1)
    t, arrivals = 0, []
    for _ in range(300):
        t += int(rng.expovariate(1 / 60e6))
        arrivals.append((t, rng.randrange(50, 3000), rng.randrange(1, 300)))
    base = T.simulate(paper_params(policy=T.SARATHI, total_pages=20000), T.StageModel(), arrivals)
    ours = T.simulate(paper_params(policy=T.THROTTLE, total_pages=20000), T.StageModel(), arrivals)
    useful = sum(p + o - 1 for _, p, o in arrivals)       # every prompt token once, every output token but the last fed back
    assert ours["preemptions"] == 0 and ours["tokens"] == useful
    assert base["tokens"] >= useful and (base["tokens"] > useful) == (base["preemptions"] > 0)
    assert ours["bubble_ppm_last_stage"] < base["bubble_ppm_last_stage"]
    assert ours["var_batch_tokens_x1000"] < base["var_batch_tokens_x1000"]
    assert ours["end_ns"] <= base["end_ns"]
