"""Pins of the page-pool oracle (oracle/kv_oracle.py) and of prefix caching inside the scheduling oracle.

None of these re-uses the oracle's own data structure as the expected value: hand-worked traces fix the placement
and eviction order of readings K3 / K4; a shadow model that stores, per page, the whole prefix a page was computed
for (a set of prefixes, no tree, no parents) fixes what a lookup must return and shows that a page found by a lookup
always holds exactly the KV of the prompt's prefix -- through evictions, re-use of page ids, preemptions and
recomputation.
"""
import random

import pytest

from oracle import kv_oracle as K
from oracle import throttle_oracle as T

PAGE = 16


def toks(*page_labels):
    """A prompt made of whole pages, page j filled with the value page_labels[j]."""
    out = []
    for v in page_labels:
        out += [v] * PAGE
    return out


def chain(pool, tokens, pages):
    """Registers pages (already held) as the successive whole pages of tokens."""
    parent = K.ROOT
    for i, pg in enumerate(pages):
        assert pool.register(parent, tokens[i * PAGE:(i + 1) * PAGE], pg)
        parent = pg


def test_free_stack_hands_out_ascending_ids_then_most_recently_returned_first():
    pool = K.PagePool(4)
    assert [pool.alloc() for _ in range(4)] == [0, 1, 2, 3] and pool.available() == 0
    pool.release([1, 2])                       # table order: 1 then 2 -> 2 lies on top
    assert pool.available() == 2
    assert pool.alloc() == 2 and pool.alloc() == 1
    pool.release([3, 0, 2])
    assert [pool.alloc() for _ in range(3)] == [2, 0, 3]


def test_free_pages_go_before_cached_ones_and_a_chain_is_evicted_from_its_end():
    pool = K.PagePool(4)
    a = toks(1, 2, 3)
    pages = [pool.alloc() for _ in range(3)]
    chain(pool, a, pages)
    pool.release(pages)
    assert pool.available() == 4               # cached pages count as idle memory (K2)
    assert pool.alloc() == 3                   # the never-used page first
    got = pool.match(a, 9)
    assert got == [0, 1, 2]                    # the content survived the release
    pool.release(got)
    assert pool.alloc() == 2                   # deepest page of the chain first (K3)
    assert pool.match(a, 9) == [0, 1]
    pool.release([0, 1])
    assert pool.alloc() == 1 and pool.match(a, 9) == [0]
    pool.release([0])
    assert pool.alloc() == 0 and pool.match(a, 9) == [] and pool.evictions == 3


def test_least_recently_released_chain_goes_first_and_a_lookup_renews_it():
    pool = K.PagePool(4)
    x, y = toks(1, 2), toks(3, 4)
    px = [pool.alloc(), pool.alloc()]
    py = [pool.alloc(), pool.alloc()]
    chain(pool, x, px)
    chain(pool, y, py)
    pool.release(px)
    pool.release(py)
    renewed = pool.match(x, 9)
    assert renewed == px
    pool.release(renewed)                      # now y is the older one
    assert [pool.alloc() for _ in range(4)] == [py[1], py[0], px[1], px[0]]


def test_a_shared_page_outlives_every_page_that_extends_it():
    pool = K.PagePool(3)
    p, c1, c2 = pool.alloc(), pool.alloc(), pool.alloc()
    assert pool.register(K.ROOT, [7] * PAGE, p)
    assert pool.register(p, [8] * PAGE, c1)
    got = pool.match(toks(7, 9), 1)            # a second request takes the shared first page ...
    assert got == [p] and pool.count[p] == 2
    assert pool.register(p, [9] * PAGE, c2)    # ... and extends it differently
    pool.release([p, c1])
    assert pool.available() == 1               # p is still held by the second request
    pool.release([p, c2])
    assert pool.available() == 3
    assert [pool.alloc() for _ in range(3)] == [c1, c2, p]


def test_lookup_stops_at_the_first_missing_page_and_respects_its_bound():
    pool = K.PagePool(8)
    a = toks(1, 2, 3, 4)
    pages = [pool.alloc() for _ in range(4)]
    chain(pool, a, pages)
    assert pool.match(toks(1, 2, 9, 4), 9) == pages[:2]          # page 3 differs: page 4 is not reachable
    assert pool.match(toks(9, 2, 3, 4), 9) == []
    assert pool.match(a, 3) == pages[:3]
    assert pool.match(a[:-1], 9) == pages[:3]                    # 63 tokens hold only 3 whole pages
    assert pool.match(toks(2), 9) == []                          # page content 2 exists, but not as a first page
    assert [pool.count[p] for p in pages] == [4, 4, 3, 1]


def test_registering_a_prefix_twice_fails_and_the_page_stays_private():
    pool = K.PagePool(3)
    p, q = pool.alloc(), pool.alloc()
    assert pool.register(K.ROOT, [5] * PAGE, p)
    assert not pool.register(K.ROOT, [5] * PAGE, q)
    pool.release([q])
    assert pool.alloc() == q                    # it went to the free stack, not to the eviction queue
    assert pool.match(toks(5), 9) == [p]


class Shadow:
    """What every page holds, written down without any tree: the full prefix it was computed for."""

    def __init__(self, total):
        self.content = [None] * total           # page -> tuple of all tokens up to the end of that page
        self.holders = [0] * total

    def live_prefixes(self):
        return {c for c in self.content if c is not None}

    def longest(self, tokens, bound):
        live, k = self.live_prefixes(), 0
        while k < min(bound, len(tokens) // PAGE) and tuple(tokens[:(k + 1) * PAGE]) in live:
            k += 1
        return k


@pytest.mark.parametrize("seed,total", [(0, 6), (1, 12), (2, 40)])
def test_random_traffic_against_a_shadow_of_page_contents(seed, total):
    rng = random.Random(seed)
    pool, sh = K.PagePool(total), Shadow(total)
    stems = [[rng.randrange(3) for _ in range(PAGE * 5)] for _ in range(3)]
    held = []                                   # (tokens, pages) of live "requests"
    for step in range(3000):
        if held and (rng.random() < 0.45 or pool.available() == 0):
            tokens, pages = held.pop(rng.randrange(len(held)))
            pool.release(pages)
            for p in pages:
                sh.holders[p] -= 1
        else:
            stem = rng.choice(stems)
            cut = rng.randrange(0, len(stem) + 1)
            tokens = stem[:cut] + [rng.randrange(3, 50) for _ in range(rng.randrange(1, 40))]
            bound = (len(tokens) - 1) // PAGE
            want = sh.longest(tokens, bound)
            pages = pool.match(tokens, bound)
            assert len(pages) == want                                              # K5 against the plain definition
            for i, p in enumerate(pages):
                assert sh.content[p] == tuple(tokens[:(i + 1) * PAGE])             # the page holds this very prefix
                sh.holders[p] += 1
            n_pages = -(-len(tokens) // PAGE)
            registering = True
            while len(pages) < n_pages and pool.available() > 0:
                p = pool.alloc()
                assert sh.holders[p] == 0                                          # never a page somebody holds
                sh.content[p] = None                                               # overwritten
                sh.holders[p] = 1
                i = len(pages)
                pages.append(p)
                if registering and (i + 1) * PAGE <= len(tokens):
                    prefix = tuple(tokens[:(i + 1) * PAGE])
                    fresh = prefix not in sh.live_prefixes()
                    ok = pool.register(pages[i - 1] if i else K.ROOT, tokens[i * PAGE:(i + 1) * PAGE], p)
                    assert ok == fresh                                             # K6
                    if ok:
                        sh.content[p] = prefix
                    else:
                        registering = False
            held.append((tokens, pages))
        assert [pool.count[p] for p in range(total)] == sh.holders
        assert pool.available() == sum(1 for h in sh.holders if h == 0)            # K2: nothing is lost
    for tokens, pages in held:
        pool.release(pages)
    assert pool.available() == total


# ---- prefix caching inside the scheduler (reading R9) --------------------------------------------------------

def params(**kw):
    base = dict(policy=T.THROTTLE, iters_t=1, max_p=4096, min_p=1, kv_thresh_bp=0, pp_depth=1, token_budget=4096,
                total_pages=64, prefix_caching=True)
    base.update(kw)
    return T.Params(**base)


def run_to_end(s, log=None):
    while True:
        got = s.next_batch()
        if got is None:
            break
        if log is not None:
            log.append(got[1])
        s.complete_batch(got[0])


def test_a_repeated_prompt_skips_its_cached_whole_pages_but_never_all_of_it():
    s = T.Scheduler(params())
    a = list(range(64))
    s.add_request(0, 64, 1, a)
    log = []
    run_to_end(s, log)
    assert log == [[(0, 64, 0)]]
    s.add_request(1, 64, 1, a)                  # 4 whole pages are cached; one token must still be computed
    s.add_request(2, 65, 1, a + [7])
    s.add_request(3, 40, 1, a[:40])
    s.add_request(4, 64, 1, a[:32] + [0] * 32)
    run_to_end(s, log)
    assert log[1] == [(1, 16, 48), (2, 1, 64), (3, 8, 32), (4, 32, 32)]
    assert s.hit_tokens == 48 + 64 + 32 + 32
    assert s.free_pages == 64


def test_pages_are_shared_not_copied_and_survive_their_first_owner():
    s = T.Scheduler(params(pp_depth=2))
    a = list(range(100, 148))
    s.add_request(0, 48, 3, a)
    bid, rows = s.next_batch()
    first = list(s.req[0].block_table)
    s.complete_batch(bid)
    s.add_request(1, 48, 2, a)
    bid, rows = s.next_batch()                  # decode row of 0 and the prompt of 1
    assert rows == [(0, 1, 48), (1, 16, 32)]
    assert s.req[1].block_table[:2] == first[:2] and s.req[1].block_table[2] not in first
    assert s.free_pages == 64 - 4 - 1           # 0 holds 3 + 1 pages, 1 adds only one of its own
    s.complete_batch(bid)
    run_to_end(s)
    assert sorted(s.finished) == [0, 1] and s.free_pages == 64


def test_without_shared_content_caching_changes_no_row_of_the_schedule():
    rng = random.Random(3)
    reqs = [(rng.randrange(1, 300), rng.randrange(1, 30)) for _ in range(60)]
    logs = []
    for caching in (False, True):
        s = T.Scheduler(params(iters_t=4, max_p=256, min_p=8, kv_thresh_bp=500, pp_depth=3, total_pages=200, prefix_caching=caching))
        log, flying, nxt = [], [], 0
        for step in range(5000):
            if nxt < len(reqs) and step % 3 == 0:
                n, o = reqs[nxt]
                s.add_request(nxt, n, o, [nxt * 1000 + j for j in range(n)])       # no two prompts share a token
                nxt += 1
            got = s.next_batch()
            if got is not None:
                log.append(got[1])
                flying.append(got[0])
            if flying and (got is None or len(flying) == 3):
                s.complete_batch(flying.pop(0))
            if nxt == len(reqs) and len(s.finished) == len(reqs):
                break
        assert len(s.finished) == len(reqs) and s.preemptions == 0     # (a restarted request would find its own pages)
        assert (s.pool.evictions > 0) == caching                          # the pool is small enough to recycle cached pages
        logs.append(log)
    assert logs[0] == logs[1]


@pytest.mark.parametrize("report", [False, True])
@pytest.mark.parametrize("seed,pages,policy", [(0, 40, T.THROTTLE), (1, 24, T.THROTTLE), (2, 30, T.SARATHI), (3, 200, T.THROTTLE)])
def test_every_cached_position_a_row_relies_on_holds_the_kv_of_that_requests_own_prefix(seed, pages, policy, report):
    """The property prefix caching must keep: row (request, n, c) reads positions 0..c-1 through its block table,
    and each must have been written for exactly this request's tokens 0..position.  The shadow KV store is keyed by
    (page, slot) and written at launch, in launch order (a pipeline runs micro-batches in order)."""
    rng = random.Random(seed)
    s = T.Scheduler(params(policy=policy, iters_t=3, max_p=96, min_p=8, kv_thresh_bp=0, pp_depth=3, token_budget=96,
                           total_pages=pages))
    stems = [[rng.randrange(5) for _ in range(200)] for _ in range(3)]
    n_req = 50
    full = {}                                   # request -> prompt followed by its (made-up) generated tokens
    store = {}
    flying, nxt, skipped, computed = [], 0, 0, 0
    for step in range(20000):
        if nxt < n_req and rng.random() < 0.3:
            stem = rng.choice(stems)
            prompt = stem[:rng.randrange(0, 160)] + [rng.randrange(5, 99) for _ in range(rng.randrange(1, 30))]
            out = rng.randrange(1, 25)
            if -(-(len(prompt) + out) // PAGE) <= pages:
                full[nxt] = prompt + [1000 + nxt * 100 + j for j in range(out)]
                s.add_request(nxt, len(prompt), out, prompt)
            else:
                full[nxt] = None
            nxt += 1
        got = s.next_batch()
        if got is not None:
            bid, rows = got
            for rid, n, c in rows:
                bt = s.req[rid].block_table
                assert len(bt) == -(-(c + n) // PAGE)
                for pos in range(c):
                    assert store[(bt[pos // PAGE], pos % PAGE)] == tuple(full[rid][:pos + 1]), (rid, pos)
                for pos in range(c, c + n):
                    store[(bt[pos // PAGE], pos % PAGE)] = tuple(full[rid][:pos + 1])
                computed += n
            flying.append((bid, rows))
        if flying and (got is None or len(flying) == 3):
            bid, rows = flying.pop(0)
            # every row reports the token that follows its last position (rows that yield none ignore it)
            s.complete_batch(bid, [full[rid][c + n] if report and c + n < len(full[rid]) else -1 for rid, n, c in rows])
        live = [r for r in full if full[r] is not None]
        if nxt == n_req and len(s.finished) == len(live) and not flying:
            break
    assert sorted(s.finished) == sorted(r for r in full if full[r] is not None)
    assert s.free_pages == pages
    assert s.hit_tokens > 0                     # the stems do get shared
    if pages <= 40:
        assert s.preemptions > 0                # and the small pools force recomputation on top


def test_a_follow_up_request_finds_the_pages_of_the_reported_answer():
    s = T.Scheduler(params(pp_depth=1))
    prompt = list(range(500, 540))                                   # 40 tokens
    answer = list(range(900, 930))                                   # 30 tokens
    s.add_request(0, 40, 30, prompt)
    step = 0
    while True:
        got = s.next_batch()
        if got is None:
            break
        bid, rows = got
        s.complete_batch(bid, [answer[step]])                        # one row per micro-batch here
        step += 1
    assert step == 30 and s.finished == [0]
    # the cache holds positions 0..68 (the last answer token was never fed back): 4 whole pages of known tokens
    follow_up = prompt + answer + list(range(100, 120))              # 90 tokens
    s.add_request(1, 90, 1, follow_up)
    assert s.next_batch()[1] == [(1, 26, 64)]
    # the same conversation when the answer was not reported: only the prompt's two whole pages are found
    s2 = T.Scheduler(params(pp_depth=1))
    s2.add_request(0, 40, 30, prompt)
    run_to_end(s2)
    s2.add_request(1, 90, 1, follow_up)
    assert s2.next_batch()[1] == [(1, 58, 32)]


def test_a_recomputed_request_finds_its_own_answer_so_far():
    """6 pages cannot hold both requests to their ends: one is preempted while decoding, and when it starts over
    its first chunk begins behind more whole pages than its prompt has -- pages that hold answer tokens and can
    only be in the tree because reported tokens are registered."""
    s = T.Scheduler(params(pp_depth=1, total_pages=6, min_p=1))
    s.add_request(0, 40, 40, list(range(1000, 1040)))               # grows to 5 pages
    s.add_request(1, 10, 30, list(range(2000, 2010)))               # grows to 3 pages
    restarts = []
    for _ in range(400):
        got = s.next_batch()
        if got is None:
            break
        bid, rows = got
        restarts += [(rid, n, c) for rid, n, c in rows if n > 1 and c > 0]     # prompts go in one chunk here unless cached
        s.complete_batch(bid, [7000 + 100 * rid + c + n for rid, n, c in rows])  # a token that depends on its position
    assert sorted(s.finished) == [0, 1] and s.preemptions > 0
    whole_prompt_pages = {0: 32, 1: 0}                              # what the prompts alone could give
    assert restarts and all(c % 16 == 0 and c > whole_prompt_pages[rid] for rid, n, c in restarts)
    assert s.free_pages == 6
