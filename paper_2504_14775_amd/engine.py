"""A serving loop on one GPU around the library's pieces: scheduler -> embedding -> stage -> final norm + vocabulary
projection -> sampler, the sampled tokens going back into the requests.

One pipeline stage holds the whole model here (one GPU), so what is shown of the paper's runtime (arxiv 2504.14775,
section 3.3) is its asynchronous side: up to #PP_depth micro-batches are enqueued before the oldest one is waited
for, so the host work of a micro-batch (scheduling, block tables, token ids: the "metadata") runs while the GPU
executes the micro-batches before it; only the sampled token ids travel back.  This module does no arithmetic on
activations: every step of the path is a call into the C ABI (binding.py, sched.py, head.py).
"""
from __future__ import annotations

from collections import deque
from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import binding, head, sched, synth

PAGE = 16


@dataclass
class Sampling:
    temperature: float = 0.0     # <= 0: greedy
    top_k: int = 0               # 0: no limit
    top_p: float = 1.0
    seed: int = 0


@dataclass
class _Request:
    tokens: List[int]            # prompt, then every token generated so far
    prompt_len: int
    max_new: int
    sampling: Sampling
    rng: np.random.Generator
    done: bool = False


@dataclass
class _Slot:
    """Buffers of one micro-batch in flight."""
    ids_host: object
    ids: object
    x: object
    out: object
    out32: object
    par_host: object             # pinned [5, max_seqs] 32-bit words: selected rows, top_k (int32), temperature, top_p, u (float32)
    par: object                  # the same on the device: one copy per micro-batch
    logits: object
    picked: object
    picked_host: object
    event: object
    staged: object               # the layers of the micro-batch are done (what the second stream waits for)
    begin: object                # timed event in front of the micro-batch (timing mode)
    batch_id: int = -1
    rows: List[Tuple[int, int, int]] = field(default_factory=list)
    takers: List[int] = field(default_factory=list)
    num_tokens: int = 0


def pick_independent(n: int, fixed: int, total: int, clash: Dict[Tuple[int, int], bool]) -> List[int]:
    """Host logic of independent_streams: indices of n of the candidates fixed .. total-1 such that no two of them,
    and none of them with one of the candidates 0 .. fixed-1, clash (clash[(i, j)], i < j).  Greedy from every starting
    candidate, first complete set wins; when no complete set exists the largest one found is filled up with the lowest
    remaining indices."""
    best: List[int] = []
    for first in range(fixed, total):
        if any(clash[(q, first)] for q in range(fixed)):
            continue
        pick = list(range(fixed)) + [first]
        for k in range(fixed, total):
            if k not in pick and len(pick) < fixed + n and not any(clash[(min(k, q), max(k, q))] for q in pick):
                pick.append(k)
        if len(pick) - fixed > len(best):
            best = pick[fixed:]
        if len(best) >= n:
            break
    rest = [k for k in range(fixed, total) if k not in best]
    return (best + rest)[:n]


def independent_streams(n: int, device: str = "cuda", candidates: int = 8, beside: Sequence = ()) -> List:
    """n streams whose kernels can run at the same time.  The runtime multiplexes streams onto a few hardware
    queues (four per process here), fixed per stream when it is made, and two streams that share a queue run their
    kernels strictly one after the other -- which of a handful of new streams collide differs from run to run.
    So: make `candidates` streams, time a short matrix-core kernel (one workgroup per eighth of the chip, 0.3 ms)
    alone and on every pair, and pick greedily n streams that overlap pairwise, and with every stream of `beside`
    (streams the caller already uses).  Falls back to the first ones when no such set exists."""
    import itertools
    import torch
    if n <= 0:
        return []
    fixed = len(beside)
    cands = list(beside) + [torch.cuda.Stream(device=device) for _ in range(max(candidates, n))]
    sink = torch.randn(1 << 12, device=device)

    def run(streams):
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for st in streams:
            st.wait_event(a)
            binding.gllm_op_peak_mfma(sink, 32, 1500, stream=st)
        for st in streams:
            torch.cuda.current_stream().wait_stream(st)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b)

    run(cands[:1])                                             # first-use costs
    alone = min(run(cands[:1]) for _ in range(3))
    clash = {(i, j): run([cands[i], cands[j]]) > 1.5 * alone for i, j in itertools.combinations(range(len(cands)), 2)}
    return [cands[k] for k in pick_independent(n, fixed, len(cands), clash)]


class Engine:
    def __init__(self, shape: synth.StageShape, vocab: int, params: sched.Params, *, max_batch_tokens: int,
                 max_batch_seqs: int, max_context: int, device: str = "cuda", max_in_flight: Optional[int] = None,
                 timing: bool = False, overlap_head: bool = True, lanes: Optional[int] = None):
        """max_in_flight: micro-batches enqueued before the oldest is waited for (default and at most #PP_depth;
        1 makes the loop synchronous).  timing: bracket every micro-batch with timed events (stats["gpu_ms"]; the
        brackets of consecutive micro-batches overlap when overlap_head is on).  overlap_head: the last-stage extras
        of a micro-batch (projection, sampler, read-back) run on a second stream, next to the layers of the
        micro-batch after it -- they only read the finished micro-batch's own output buffer.  lanes (default 2 where
        #PP_depth allows, at most #PP_depth): 2 runs the
        layers of consecutive micro-batches on two streams through two stage objects (each with its own workspace,
        sharing one set of weights, both bound to the one KV pool): micro-batches in flight never share a
        request and only read shared prefix pages, so they are independent, and the gaps between the dependent
        kernels of one are filled by the kernels of the other."""
        import torch
        self.torch = torch
        self.shape, self.vocab, self.params, self.device = shape, vocab, params, device
        self.max_tokens, self.max_seqs, self.max_context = max_batch_tokens, max_batch_seqs, max_context
        self.max_blocks = -(-max_context // PAGE)
        self.sched = sched.Scheduler(params)
        if lanes is None:
            lanes = min(2, max(1, params.pp_depth))
        if not 1 <= lanes <= max(1, params.pp_depth):
            raise ValueError("lanes must be between 1 and #PP_depth")
        self.stages, self._ws = [], []
        for _ in range(lanes):
            st = binding.Stage(binding.make_config(shape, max_batch_tokens, max_batch_seqs, self.max_blocks, max_context))
            ws = torch.empty(st.workspace_bytes(), dtype=torch.uint8, device=device)
            st.bind_workspace(ws)
            self.stages.append(st)
            self._ws.append(ws)
        self.stage = self.stages[0]
        if lanes > 1:
            # with a second lane the stage's own fork (prefill attention on a side stream) only adds streams that
            # compete for the few hardware queues: measured 27.3k tokens/s with it against 29.0k without
            for st in self.stages:
                st.set_option("overlap_attention", 0)
        # streams that do not share a hardware queue: the lanes first, then the one for the last-stage extras
        own = independent_streams((lanes if lanes > 1 else 0) + (1 if overlap_head else 0), device,
                                  beside=() if lanes > 1 else (torch.cuda.current_stream(),))
        self.lane_streams = own[:lanes] if lanes > 1 else [None]
        self.launched = 0
        self.head = head.Head(shape.hidden, vocab, max_batch_seqs, shape.rms_eps, device=device)
        n_el = shape.num_layers * synth.pool_elems_per_layer(shape, params.total_pages)
        self.k_pool = torch.zeros(n_el, dtype=torch.bfloat16, device=device)
        self.v_pool = torch.zeros(n_el, dtype=torch.bfloat16, device=device)
        for st in self.stages:
            st.bind_kv_pool(self.k_pool, self.v_pool, params.total_pages)
        self.table = None
        self.requests: Dict[int, _Request] = {}
        self.flying: deque = deque()
        self.timing = timing
        self.tail = own[-1] if overlap_head else None
        depth = params.pp_depth if max_in_flight is None else max(1, min(max_in_flight, params.pp_depth))
        self.free_slots = [self._make_slot() for _ in range(depth)]
        self.observer: Optional[Callable] = None     # tests: called with the slot of every retired micro-batch
        self.stats = {"micro_batches": 0, "tokens_computed": 0, "tokens_generated": 0, "gpu_ms": 0.0}

    def _make_slot(self) -> _Slot:
        t, dev, H = self.torch, self.device, self.shape.hidden
        T, S = self.max_tokens, self.max_seqs
        pin = lambda *shape, dtype: t.empty(*shape, dtype=dtype, pin_memory=True)
        return _Slot(
            ids_host=pin(T, dtype=t.int32), ids=t.empty(T, dtype=t.int32, device=dev),
            x=t.empty(T, H, dtype=t.bfloat16, device=dev), out=t.empty(T, H, dtype=t.bfloat16, device=dev),
            out32=t.empty(T, H, dtype=t.float32, device=dev),
            par_host=pin(5, S, dtype=t.int32).zero_(), par=t.zeros(5, S, dtype=t.int32, device=dev),
            logits=t.empty(S, self.head.padded_vocab, dtype=t.float32, device=dev),
            picked=t.empty(S, dtype=t.int32, device=dev), picked_host=pin(S, dtype=t.int32),
            event=t.cuda.Event(enable_timing=self.timing), staged=t.cuda.Event(), begin=t.cuda.Event(enable_timing=True) if self.timing else None)

    # ---- set-up -----------------------------------------------------------------------------------------------
    def load(self, layers: Sequence[Dict[str, object]], embedding_table, final_norm_gain, w_vocab) -> None:
        """layers: per layer the device tensors gllm_stage_load_layer takes; embedding_table: bf16 [vocab, hidden];
        final_norm_gain: bf16 [hidden]; w_vocab: bf16 [vocab, hidden].  The table is used in place (keep it alive)."""
        for l, w in enumerate(layers):
            self.stages[0].load_layer(l, w)
        self.torch.cuda.synchronize()
        for st in self.stages[1:]:
            st.share_weights(self.stages[0])
        self.head.load(final_norm_gain, w_vocab)
        self.table = embedding_table
        self.torch.cuda.synchronize()

    def add_request(self, request_id: int, prompt: Sequence[int], max_new_tokens: int, sampling: Optional[Sampling] = None) -> None:
        if len(prompt) + max_new_tokens > self.max_context:
            raise ValueError("prompt + max_new_tokens exceeds max_context")
        sp = sampling or Sampling()
        self.sched.add_request(request_id, len(prompt), max_new_tokens,
                               tokens=list(prompt) if self.params.prefix_caching else None)
        self.requests[request_id] = _Request(list(prompt), len(prompt), max_new_tokens, sp, np.random.default_rng(sp.seed))

    # ---- the loop ---------------------------------------------------------------------------------------------
    def _launch(self) -> bool:
        """Schedules one micro-batch and enqueues all of its GPU work; False when nothing could be scheduled."""
        if not self.free_slots:
            return False
        got = self.sched.next_batch()
        if got is None:
            return False
        t = self.torch
        bid, rows = got
        nt = np.fromiter((n for _, n, _ in rows), dtype=np.int32, count=len(rows))
        cl = np.fromiter((c for _, _, c in rows), dtype=np.int32, count=len(rows))
        T = int(nt.sum())
        if T > self.max_tokens or len(rows) > self.max_seqs:
            raise RuntimeError(f"micro-batch of {T} tokens / {len(rows)} rows exceeds the engine's sizes")
        bt = self.sched.block_tables(bid, len(rows), self.max_blocks)
        slot = self.free_slots.pop()
        ids = slot.ids_host.numpy()
        at = 0
        takers = []
        for i, (rid, n, c) in enumerate(rows):
            r = self.requests[rid]
            ids[at:at + n] = r.tokens[c:c + n]
            at += n
            if c + n == len(r.tokens):                     # the row's last token is the newest one: it yields the next
                takers.append(i)
        m = len(takers)
        if m:
            ends = np.cumsum(nt) - 1
            words = slot.par_host.numpy()
            reals = words.view(np.float32)
            words[0, :m] = ends[takers]
            for j, i in enumerate(takers):
                r = self.requests[rows[i][0]]
                words[1, j] = r.sampling.top_k
                reals[2, j], reals[3, j] = r.sampling.temperature, r.sampling.top_p
                reals[4, j] = r.rng.random(dtype=np.float32) if r.sampling.temperature > 0 else 0.0
        lane = self.launched % len(self.stages)
        self.launched += 1
        main = self.lane_streams[lane] if self.lane_streams[lane] is not None else t.cuda.current_stream()
        with t.cuda.stream(main):
            if self.timing:
                slot.begin.record()
            slot.ids[:T].copy_(slot.ids_host[:T], non_blocking=True)
            head.gllm_op_embedding(slot.ids[:T], self.table, slot.x[:T])
            self.stages[lane].forward(nt, cl, bt, slot.x, slot.out, slot.out32)
            if m and self.tail is not None:
                slot.staged.record()
            if not m:
                slot.event.record()
        if m:
            if self.tail is not None:
                self.tail.wait_event(slot.staged)
            with t.cuda.stream(self.tail if self.tail is not None else main):
                slot.par.copy_(slot.par_host, non_blocking=True)
                reals_dev = slot.par.view(t.float32)
                self.head.logits(slot.out32[:T], slot.par[0, :m], slot.logits[:m])
                head.gllm_op_sample(slot.logits[:m], self.vocab, reals_dev[2, :m], slot.par[1, :m], reals_dev[3, :m],
                                    reals_dev[4, :m], slot.picked[:m])
                slot.picked_host[:m].copy_(slot.picked[:m], non_blocking=True)
                slot.event.record()
        slot.batch_id, slot.rows, slot.takers, slot.num_tokens = bid, rows, takers, T
        self.flying.append(slot)
        self.stats["micro_batches"] += 1
        self.stats["tokens_computed"] += T
        return True

    def _retire(self) -> List[Tuple[int, int, bool]]:
        """Waits for the oldest micro-batch; returns (request id, new token, request ended) per token it produced."""
        slot = self.flying.popleft()
        slot.event.synchronize()
        if self.timing:
            self.stats["gpu_ms"] += slot.begin.elapsed_time(slot.event)
        picked = slot.picked_host.numpy()
        news = []
        for j, i in enumerate(slot.takers):
            rid = slot.rows[i][0]
            self.requests[rid].tokens.append(int(picked[j]))
            news.append(rid)
        if self.observer is not None:
            self.observer(slot)
        row_tokens = np.full(len(slot.rows), -1, dtype=np.int32)      # reported, so that answers enter the prefix cache
        row_tokens[slot.takers] = picked[:len(slot.takers)]
        ended = set(self.sched.complete_batch(slot.batch_id, row_tokens))
        for rid in ended:
            self.requests[rid].done = True
        self.stats["tokens_generated"] += len(news)
        self.free_slots.append(slot)
        return [(rid, self.requests[rid].tokens[-1], rid in ended) for rid in news]

    def step(self) -> List[Tuple[int, int, bool]]:
        """Enqueues micro-batches while the scheduler yields some and the pipeline has room, then retires the oldest
        one.  Returns the tokens that became known; empty when nothing is in flight and nothing can be scheduled."""
        while self._launch():
            pass
        return self._retire() if self.flying else []

    def run(self) -> Dict[int, List[int]]:
        """Runs until every request has ended; returns the generated tokens per request id."""
        while any(not r.done for r in self.requests.values()):
            launched = False
            while self._launch():
                launched = True
            if self.flying:
                self._retire()
            elif not launched:
                raise RuntimeError("the scheduler cannot make progress (pool too small for the oldest request?)")
        return {rid: r.tokens[r.prompt_len:] for rid, r in self.requests.items()}

    def close(self) -> None:
        self.torch.cuda.synchronize()
        self.head.destroy()
        for st in reversed(self.stages):             # the borrowers first, the owner of the weights last
            st.destroy()
