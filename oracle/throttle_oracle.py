"""TEST INFRASTRUCTURE -- plain Python statement of the paper's micro-batch scheduling rules.

Only tests/ (and the bench scripts' baseline legs) may import this module; the library never does.

What is stated here, with the passage of arxiv 2504.14775 each part follows:

* prefill_budget():  Prefill Token Throttling, section 3.1: Eq. 1 (throttling by tokens awaiting prefill, WT),
  Eq. 2 (throttling by KV-cache idle rate, UT), the idle-rate threshold, and their combination Eq. 3.
* decode_budget():   Decode Token Throttling, section 3.2, Eq. 4.
* Scheduler:         the iteration-level scheduler that turns the two budgets into one merged micro-batch
  (opening of section 3: prefill and decode tokens are scheduled separately, then merged), with the chunked-prefill
  baseline of section 2.2 (all decode requests first, then prefill chunks up to a fixed token budget) as the
  other policy.  KV pages are assigned before a micro-batch runs and released when a request ends (caption of
  the prefill case study, section 3.1); at most pipeline-depth micro-batches are in flight (section 3.2).
* simulate():        a pipeline of `pp_depth` equal stages fed by that scheduler, with a linear stage-time model.
  Not from the paper: a measuring device for bubbles and token-count variance.

Readings where the paper is silent or at odds with itself (each is a parameter-free choice stated once):
  R1  #WP/#T and #RD/#PP_depth are rounded up; #MaxP x (idle fraction) is rounded down.
  R2  idle rate below the threshold suspends prefill (#P = 0), as the text of "Threshold" says, although Eq. 3
      alone would still give #MinP.  At or above the threshold Eq. 3 applies.
  R3  #P never exceeds #WP, nor #MaxP (Eq. 3 bounds it by #MaxP only through its idle-rate term; without that
      term Eq. 1's bound is used), nor what the free pages can hold.
  R4  the idle rate is the one at the start of the scheduling step (before this step's decode pages).
  R5  a request is in at most one micro-batch in flight; #RD counts every request in its decode phase,
      in flight or not; decode requests are taken in least-recently-run order.
  R6  a decode request that needs a page when none is free preempts the most recently admitted idle decode
      request (pages released, the request re-enters the waiting queue at its front with its generated tokens
      appended to its prompt: recomputation, section 3.1 "Threshold"); with no such victim it takes the pages
      of the last waiting request that holds some and is not in flight (that request starts over); with no
      victim at all it waits.  The first schedulable waiting request, when no page is left for it, likewise
      takes the pages of waiting requests behind it, last first.  Without these two rules a small pool can
      fill up with half-prefilled prompts and stop for good.
  R7  all arithmetic is integer; the threshold is given in 1/10000.
  R8  pages come from the page pool of kv_oracle.py: a last-in-first-out free stack that first hands out 0, 1,
      2, ...; a request's pages return to it in block-table order.  (Placement policy is not the paper's
      subject; fixed here so that two implementations can be compared id by id.)
  R9  with prefix caching (section 3.4 lists it among the integrated techniques; off in the paper's runs,
      section 4.1) a request that is about to receive its first chunk, or starts over after a preemption, first
      looks its prompt up in the pool and skips the whole pages found, leaving at least one token to compute;
      whole pages of known tokens are registered when the micro-batch that fills them has left the last stage,
      until one registration fails; pages nobody holds that still carry a registered prefix count as idle KV
      memory in Eq. 2 / Eq. 3 (they are reclaimed on demand).  Known tokens are the prompt as given on arrival
      and the generated tokens the caller reports with complete_batch() (a follow-up request that repeats the
      conversation so far then finds the answer's pages too); the newest token is known one step before its KV
      is in the cache, so a page is registered when the step that computes its last position has completed.
"""
from collections import deque
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

from .kv_oracle import ROOT, PagePool

PAGE = 16
SARATHI, THROTTLE = 0, 1
BIG = 1 << 60


@dataclass
class Params:
    policy: int = THROTTLE
    iters_t: int = 8            # #T
    max_p: int = 2048           # #MaxP
    min_p: int = 32             # #MinP
    kv_thresh_bp: int = 500     # KV_thresh in 1/10000 (0.05)
    pp_depth: int = 4           # #PP_depth
    token_budget: int = 2048    # chunked-prefill baseline: tokens per micro-batch
    use_wt: bool = True
    use_ut: bool = True
    total_pages: int = 4096
    prefix_caching: bool = False


def ceil_div(a: int, b: int) -> int:
    return -(-a // b)


def prefill_budget(p: Params, wp: int, free_pages: int) -> int:
    """#P of Eq. 3 (readings R1-R3), from the tokens awaiting prefill and the free pages."""
    if wp <= 0:
        return 0
    if free_pages * 10000 < p.kv_thresh_bp * p.total_pages:      # idle rate below the threshold
        return 0
    wt = ceil_div(wp, p.iters_t) if p.use_wt else BIG
    if p.use_ut:
        ut = (p.max_p * (free_pages * 10000 - p.kv_thresh_bp * p.total_pages)) // ((10000 - p.kv_thresh_bp) * p.total_pages)
    else:
        ut = BIG
    n = max(min(wt, ut, p.max_p), p.min_p)
    return min(n, wp)


def decode_budget(p: Params, rd: int) -> int:
    """#D of Eq. 4 (reading R1)."""
    return ceil_div(rd, p.pp_depth)


@dataclass
class Request:
    rid: int
    prompt_len: int
    output_len: int
    prefilled: int = 0      # prompt tokens whose KV is in the cache (completed chunks)
    generated: int = 0      # output tokens produced so far
    pages: int = 0
    in_flight: bool = False
    chunk: int = 0          # tokens of the chunk in flight
    admitted: int = -1      # order of entering the decode phase (for R6)
    block_table: list = None
    tokens: Optional[list] = None   # known token ids from position 0 on: the prompt, then reported output tokens (R9)
    registered: int = 0             # leading pages of the block table that are in the pool's tree
    registering: bool = True


class Scheduler:
    def __init__(self, params: Params):
        self.p = params
        self.req: Dict[int, Request] = {}
        self.waiting: deque = deque()        # request ids with prompt tokens left, FIFO
        self.ready: deque = deque()          # decode requests not in flight, least recently run first
        self.n_decode = 0                    # requests in the decode phase (#RD)
        self.pool = PagePool(params.total_pages)                              # R8
        self.in_flight: Dict[int, List[Tuple[int, int, int, bool]]] = {}
        self.next_bid = 0
        self.admit_counter = 0
        self.finished: List[int] = []
        self.preemptions = 0
        self.hit_tokens = 0                  # prompt tokens skipped thanks to the prefix cache

    @property
    def free_pages(self) -> int:
        return self.pool.available()

    def _take(self, r: Request, need: int) -> None:
        for _ in range(need):
            r.block_table.append(self.pool.alloc())
        r.pages += need

    def _release(self, r: Request) -> None:
        self.pool.release(r.block_table)
        r.block_table = []
        r.pages = 0
        r.registered = 0
        r.registering = True

    def _lookup(self, r: Request) -> None:
        """R9: the cached whole pages of the prompt become the start of the block table."""
        found = self.pool.match(r.tokens, (r.prompt_len - 1) // PAGE)
        r.block_table = list(found)
        r.pages = r.registered = len(found)
        r.prefilled = len(found) * PAGE
        self.hit_tokens += r.prefilled

    def _register(self, r: Request, in_cache: int) -> None:
        """R9: whole pages among the first in_cache positions (those whose KV has been computed) whose tokens are
        known enter the tree."""
        full = min(in_cache, len(r.tokens)) // PAGE
        while r.registering and r.registered < full:
            i = r.registered
            parent = r.block_table[i - 1] if i > 0 else ROOT
            if self.pool.register(parent, r.tokens[i * PAGE:(i + 1) * PAGE], r.block_table[i]):
                r.registered += 1
            else:
                r.registering = False

    # ---- state -------------------------------------------------------------------------------------------
    def add_request(self, rid: int, prompt_len: int, output_len: int, tokens: Optional[Sequence[int]] = None) -> None:
        assert rid not in self.req and prompt_len >= 1 and output_len >= 1
        assert tokens is None or len(tokens) == prompt_len
        keep = list(tokens) if tokens is not None and self.p.prefix_caching else None
        self.req[rid] = Request(rid, prompt_len, output_len, block_table=[], tokens=keep)
        self.waiting.append(rid)

    def tokens_waiting(self) -> int:
        """#WP: prompt tokens not yet handed to a micro-batch."""
        return sum(self.req[r].prompt_len - self.req[r].prefilled - self.req[r].chunk for r in self.waiting)

    # ---- one scheduling step -----------------------------------------------------------------------------
    def next_batch(self) -> Optional[Tuple[int, List[Tuple[int, int, int]]]]:
        """Forms the next micro-batch: (batch id, [(request id, new tokens, cached length)]), decode rows first;
        None when the pipeline is full or nothing can be scheduled."""
        p = self.p
        if len(self.in_flight) >= p.pp_depth:
            return None
        free_at_start = self.free_pages                                       # R4
        entries: List[Tuple[int, int, int, bool]] = []
        # decode rows
        quota = decode_budget(p, self.n_decode) if p.policy == THROTTLE else p.token_budget
        while quota > 0 and self.ready:
            rid = self.ready[0]
            r = self.req[rid]
            cached = r.prompt_len + r.generated - 1
            need = ceil_div(cached + 1, PAGE) - r.pages
            while need > self.free_pages:                                     # R6
                victim = None
                for cand in self.ready:
                    if cand != rid and (victim is None or self.req[cand].admitted > self.req[victim].admitted):
                        victim = cand
                if victim is not None:
                    self._preempt(victim)
                elif not self._reset_last_waiting(None):
                    break
            if need > self.free_pages:
                break
            self.ready.popleft()
            self._take(r, need)
            r.in_flight = True
            entries.append((rid, 1, cached, True))
            quota -= 1
        n_dec = len(entries)
        # prefill chunks
        wp = self.tokens_waiting()
        if p.policy == THROTTLE:
            budget = prefill_budget(p, wp, free_at_start)
        else:
            budget = min(max(p.token_budget - n_dec, 0), wp)
        for rid in list(self.waiting):
            if budget <= 0:
                break
            r = self.req[rid]
            if r.in_flight:
                continue
            if r.tokens is not None and r.prefilled == 0 and r.pages == 0:
                self._lookup(r)
            c = r.prefilled
            n = min(r.prompt_len - c, budget)
            fit = (r.pages + self.free_pages) * PAGE - c                      # R3: what the free pages can hold
            while fit <= 0 and self._reset_last_waiting(rid):                 # R6
                fit = (r.pages + self.free_pages) * PAGE - c
            if fit <= 0:
                break
            n = min(n, fit)
            self._take(r, ceil_div(c + n, PAGE) - r.pages)
            r.in_flight = True
            r.chunk = n
            entries.append((rid, n, c, False))
            budget -= n
        if not entries:
            return None
        bid = self.next_bid
        self.next_bid += 1
        self.in_flight[bid] = entries
        return bid, [(rid, n, c) for rid, n, c, _ in entries]

    def _reset_last_waiting(self, after: Optional[int]) -> bool:
        """Releases the pages of the last waiting request that holds pages and is not in flight (only requests
        behind `after` in the queue when that is given).  The request stays where it is and starts over."""
        ids = list(self.waiting)
        if after is not None:
            ids = ids[ids.index(after) + 1:]
        for cand in reversed(ids):
            r = self.req[cand]
            if not r.in_flight and r.pages > 0:
                self._release(r)
                r.prefilled = 0
                self.preemptions += 1
                return True
        return False

    def _preempt(self, rid: int) -> None:
        r = self.req[rid]
        self.ready.remove(rid)
        self.n_decode -= 1
        self._release(r)
        r.prompt_len += r.generated
        r.output_len -= r.generated
        r.generated = 0
        r.prefilled = 0
        r.admitted = -1
        self.waiting.appendleft(rid)
        self.preemptions += 1

    def complete_batch(self, bid: int, new_tokens: Optional[Sequence[int]] = None) -> List[int]:
        """The micro-batch has left the last stage.  new_tokens: per row the token it produced (ignored for rows
        that produce none; negative = not reported).  Returns the ids of the requests that ended."""
        done = []
        for i, (rid, n, c, is_decode) in enumerate(self.in_flight.pop(bid)):
            r = self.req[rid]
            r.in_flight = False
            if is_decode:
                r.generated += 1
            else:
                r.chunk = 0
                r.prefilled += n
                if r.prefilled < r.prompt_len:
                    if r.tokens is not None:
                        self._register(r, r.prefilled)
                    continue
                self.waiting.remove(rid)
                r.generated = 1                      # the last chunk yields the first output token
                r.admitted = self.admit_counter
                self.admit_counter += 1
                self.n_decode += 1
            if r.tokens is not None:
                in_cache = r.prompt_len + r.generated - 1        # the newest token's KV is not computed yet
                if new_tokens is not None and new_tokens[i] >= 0 and len(r.tokens) == in_cache:
                    r.tokens.append(int(new_tokens[i]))
                self._register(r, in_cache)
            if r.generated >= r.output_len:
                self.n_decode -= 1
                self._release(r)
                done.append(rid)
                self.finished.append(rid)
            else:
                self.ready.append(rid)
        return done


# ---- pipeline simulation ------------------------------------------------------------------------------------
@dataclass
class StageModel:
    """Time of one stage for one micro-batch, in ns: base + per new token + per cached token read by decode rows
    + per (query row x key) pair of prefill attention / 1024."""
    base_ns: int = 300_000
    token_ns: int = 33_000
    decode_ctx_ns: int = 13
    prefill_pair_ns_per_1024: int = 120

    def stage_ns(self, entries) -> int:
        t = self.base_ns
        pairs = 0
        for _, n, c in entries:
            t += n * self.token_ns
            if n == 1:
                t += (c + 1) * self.decode_ctx_ns
            else:
                pairs += n * c + n * (n + 1) // 2
        return t + pairs * self.prefill_pair_ns_per_1024 // 1024


def simulate(params: Params, model: StageModel, arrivals: List[Tuple[int, int, int]]):
    """arrivals: [(arrival time ns, prompt_len, output_len[, prompt tokens])] sorted by time; ids are their indices.
    Stage s of micro-batch j starts when stage s-1 of j and stage s of j-1 are both done.  The scheduler runs
    whenever stage 0 is free, fewer than pp_depth micro-batches are in flight and something can be scheduled.
    Returns a dict of integers (times in ns)."""
    sched = Scheduler(params)
    pp = params.pp_depth
    stage_free = [0] * pp
    busy = [0] * pp
    completions: List[Tuple[int, int]] = []          # (finish time, batch id), kept sorted by (time, bid)
    now = 0
    nxt = 0
    first_token = {}
    finish = {}
    batch_tokens: List[int] = []
    n = len(arrivals)
    while len(finish) < n:
        while nxt < n and arrivals[nxt][0] <= now:
            sched.add_request(nxt, *arrivals[nxt][1:])
            nxt += 1
        while completions and completions[0][0] <= now:
            t, bid = completions.pop(0)
            entries = list(sched.in_flight[bid])
            for rid in sched.complete_batch(bid):
                finish[rid] = t
            for rid, cnt, c, is_dec in entries:      # the chunk that completes a prompt yields the first token
                r = sched.req[rid]
                if not is_dec and rid not in first_token and r.prefilled >= r.prompt_len:
                    first_token[rid] = t
        if len(finish) >= n:
            break
        progressed = False
        if stage_free[0] <= now:
            got = sched.next_batch()
            if got is not None:
                bid, entries = got
                dt = model.stage_ns(entries)
                t = now
                for s in range(pp):
                    t = max(t, stage_free[s]) + dt
                    stage_free[s] = t
                    busy[s] += dt
                completions.append((t, bid))
                completions.sort()
                batch_tokens.append(sum(e[1] for e in entries))
                progressed = True
        if progressed:
            continue
        cands = []
        if nxt < n:
            cands.append(arrivals[nxt][0])
        if completions:
            cands.append(completions[0][0])
        if stage_free[0] > now:
            cands.append(stage_free[0])
        cands = [c for c in cands if c > now]
        if not cands:
            raise RuntimeError("simulation cannot advance")
        now = min(cands)
    end = max(finish.values())
    nb = len(batch_tokens)
    mean_x1000 = sum(batch_tokens) * 1000 // nb
    var_x1000 = sum((1000 * b - mean_x1000) ** 2 for b in batch_tokens) // nb // 1000
    return {
        "end_ns": end,
        "batches": nb,
        "tokens": sum(batch_tokens),
        "busy_ns_last_stage": busy[pp - 1],
        "bubble_ppm_last_stage": (end - busy[pp - 1]) * 1_000_000 // end,
        "mean_batch_tokens_x1000": mean_x1000,
        "var_batch_tokens_x1000": var_x1000,
        "sum_ttft_ns": sum(first_token[i] - arrivals[i][0] for i in range(n)),
        "sum_e2e_ns": sum(finish[i] - arrivals[i][0] for i in range(n)),
        "preemptions": sched.preemptions,
        "prefix_hit_tokens": sched.hit_tokens,
    }
