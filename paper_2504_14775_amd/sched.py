"""ctypes binding of the micro-batch scheduler (include/gllm_sched.h): argument marshalling only."""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

from .binding import GLLM_OK, GllmError, load_host_library

EXPORTS = [
    "gllm_sched_prefill_budget", "gllm_sched_decode_budget", "gllm_sched_create", "gllm_sched_destroy",
    "gllm_sched_add_request", "gllm_sched_add_request_tokens", "gllm_sched_next_batch", "gllm_sched_batch_block_tables",
    "gllm_sched_complete_batch", "gllm_sched_complete_batch_tokens", "gllm_sched_get_state", "gllm_sched_simulate", "gllm_sched_simulate_tokens",
]

CHUNKED_PREFILL, TOKEN_THROTTLING = 0, 1


class gllm_sched_params(C.Structure):
    _fields_ = [("policy", C.c_int32), ("iters_t", C.c_int32), ("max_p", C.c_int32), ("min_p", C.c_int32),
                ("kv_thresh_bp", C.c_int32), ("pp_depth", C.c_int32), ("token_budget", C.c_int32),
                ("use_wt", C.c_int32), ("use_ut", C.c_int32), ("prefix_caching", C.c_int32), ("total_pages", C.c_int64)]


class gllm_sched_state(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("tokens_waiting", "decode_requests", "free_pages", "batches_in_flight",
                                         "waiting_requests", "preemptions", "idle_cached_pages", "prefix_hit_tokens",
                                         "evictions")]


class gllm_stage_time_model(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("base_ns", "token_ns", "decode_ctx_ns", "prefill_pair_ns_per_1024")]


SIM_FIELDS = ("end_ns", "batches", "tokens", "busy_ns_last_stage", "bubble_ppm_last_stage", "mean_batch_tokens_x1000",
              "var_batch_tokens_x1000", "sum_ttft_ns", "sum_e2e_ns", "preemptions", "prefix_hit_tokens")


class gllm_sim_result(C.Structure):
    _fields_ = [(n, C.c_int64) for n in SIM_FIELDS]


@dataclass
class Params:
    policy: int = TOKEN_THROTTLING
    iters_t: int = 8
    max_p: int = 2048
    min_p: int = 32
    kv_thresh_bp: int = 500
    pp_depth: int = 4
    token_budget: int = 2048
    use_wt: bool = True
    use_ut: bool = True
    total_pages: int = 4096
    prefix_caching: bool = False

    def c(self) -> gllm_sched_params:
        return gllm_sched_params(self.policy, self.iters_t, self.max_p, self.min_p, self.kv_thresh_bp, self.pp_depth,
                                 self.token_budget, int(self.use_wt), int(self.use_ut), int(self.prefix_caching), self.total_pages)


_ready = False


def _lib():
    global _ready
    lib = load_host_library()
    if not _ready:
        i32, i64, vp = C.c_int32, C.c_int64, C.c_void_p
        P = C.POINTER
        lib.gllm_sched_prefill_budget.restype = i64
        lib.gllm_sched_prefill_budget.argtypes = [P(gllm_sched_params), i64, i64]
        lib.gllm_sched_decode_budget.restype = i64
        lib.gllm_sched_decode_budget.argtypes = [P(gllm_sched_params), i64]
        lib.gllm_sched_create.restype = i32
        lib.gllm_sched_create.argtypes = [P(gllm_sched_params), P(vp)]
        lib.gllm_sched_destroy.restype = None
        lib.gllm_sched_destroy.argtypes = [vp]
        lib.gllm_sched_add_request.restype = i32
        lib.gllm_sched_add_request.argtypes = [vp, i64, i32, i32]
        lib.gllm_sched_add_request_tokens.restype = i32
        lib.gllm_sched_add_request_tokens.argtypes = [vp, i64, P(i32), i32, i32]
        lib.gllm_sched_next_batch.restype = i32
        lib.gllm_sched_next_batch.argtypes = [vp, P(i64), P(i64), P(i32), P(i32), i32, P(i32)]
        lib.gllm_sched_batch_block_tables.restype = i32
        lib.gllm_sched_batch_block_tables.argtypes = [vp, i64, P(i32), i32]
        lib.gllm_sched_complete_batch.restype = i32
        lib.gllm_sched_complete_batch.argtypes = [vp, i64, P(i64), i32, P(i32)]
        lib.gllm_sched_complete_batch_tokens.restype = i32
        lib.gllm_sched_complete_batch_tokens.argtypes = [vp, i64, P(i32), i32, P(i64), i32, P(i32)]
        lib.gllm_sched_get_state.restype = i32
        lib.gllm_sched_get_state.argtypes = [vp, P(gllm_sched_state)]
        lib.gllm_sched_simulate.restype = i32
        lib.gllm_sched_simulate.argtypes = [P(gllm_sched_params), P(gllm_stage_time_model), P(i64), P(i32), P(i32), i64,
                                            P(gllm_sim_result)]
        lib.gllm_sched_simulate_tokens.restype = i32
        lib.gllm_sched_simulate_tokens.argtypes = [P(gllm_sched_params), P(gllm_stage_time_model), P(i64), P(i32), P(i32), P(i32),
                                                   i64, P(gllm_sim_result)]
        _ready = True
    return lib


def gllm_sched_prefill_budget(params: Params, wp: int, free_pages: int) -> int:
    cp = params.c()
    return int(_lib().gllm_sched_prefill_budget(C.byref(cp), wp, free_pages))


def gllm_sched_decode_budget(params: Params, rd: int) -> int:
    cp = params.c()
    return int(_lib().gllm_sched_decode_budget(C.byref(cp), rd))


def _ptr(a: np.ndarray, t):
    return a.ctypes.data_as(C.POINTER(t))


class Scheduler:
    def __init__(self, params: Params):
        self.lib = _lib()
        self.params = params
        h = C.c_void_p()
        cp = params.c()
        st = self.lib.gllm_sched_create(C.byref(cp), C.byref(h))
        if st != GLLM_OK:
            raise GllmError(st, "gllm_sched_create")
        self.handle = h
        self._count = 0

    def __del__(self):
        if getattr(self, "handle", None):
            self.lib.gllm_sched_destroy(self.handle)
            self.handle = None

    def _check(self, st: int, what: str) -> None:
        if st != GLLM_OK:
            raise GllmError(st, what)

    def add_request(self, request_id: int, prompt_len: int, output_len: int, tokens=None) -> None:
        if tokens is None:
            self._check(self.lib.gllm_sched_add_request(self.handle, request_id, prompt_len, output_len), "gllm_sched_add_request")
        else:
            t = np.ascontiguousarray(tokens, dtype=np.int32)
            if t.shape != (prompt_len,):
                raise ValueError("tokens must hold prompt_len ids")
            self._check(self.lib.gllm_sched_add_request_tokens(self.handle, request_id, _ptr(t, C.c_int32), prompt_len, output_len),
                        "gllm_sched_add_request_tokens")
        self._count += 1

    def next_batch(self, capacity: Optional[int] = None) -> Optional[Tuple[int, List[Tuple[int, int, int]]]]:
        cap = self._count if capacity is None else capacity
        ids = np.empty(max(cap, 1), dtype=np.int64)
        nt = np.empty(max(cap, 1), dtype=np.int32)
        cl = np.empty(max(cap, 1), dtype=np.int32)
        bid, n = C.c_int64(-1), C.c_int32(0)
        self._check(self.lib.gllm_sched_next_batch(self.handle, C.byref(bid), _ptr(ids, C.c_int64), _ptr(nt, C.c_int32),
                                                   _ptr(cl, C.c_int32), cap, C.byref(n)), "gllm_sched_next_batch")
        if n.value == 0:
            return None
        return bid.value, [(int(ids[i]), int(nt[i]), int(cl[i])) for i in range(n.value)]

    def block_tables(self, batch_id: int, num_rows: int, stride: int) -> np.ndarray:
        bt = np.empty((num_rows, stride), dtype=np.int32)
        self._check(self.lib.gllm_sched_batch_block_tables(self.handle, batch_id, _ptr(bt, C.c_int32), stride),
                    "gllm_sched_batch_block_tables")
        return bt

    def complete_batch(self, batch_id: int, row_tokens=None, capacity: Optional[int] = None) -> List[int]:
        """row_tokens: per row of the micro-batch the token it produced (negative: none / not reported)."""
        cap = self._count if capacity is None else capacity
        out = np.empty(max(cap, 1), dtype=np.int64)
        n = C.c_int32(0)
        if row_tokens is None:
            self._check(self.lib.gllm_sched_complete_batch(self.handle, batch_id, _ptr(out, C.c_int64), cap, C.byref(n)),
                        "gllm_sched_complete_batch")
        else:
            t = np.ascontiguousarray(row_tokens, dtype=np.int32)
            self._check(self.lib.gllm_sched_complete_batch_tokens(self.handle, batch_id, _ptr(t, C.c_int32), len(t),
                                                                  _ptr(out, C.c_int64), cap, C.byref(n)),
                        "gllm_sched_complete_batch_tokens")
        return [int(x) for x in out[:n.value]]

    def state(self) -> dict:
        st = gllm_sched_state()
        self._check(self.lib.gllm_sched_get_state(self.handle, C.byref(st)), "gllm_sched_get_state")
        return {n: int(getattr(st, n)) for n, _ in gllm_sched_state._fields_}


def gllm_sched_simulate(params: Params, model: Tuple[int, int, int, int], arrivals) -> dict:
    """arrivals: sequence of (arrival ns, prompt_len, output_len[, prompt token ids]), ascending in time."""
    a = np.ascontiguousarray([x[0] for x in arrivals], dtype=np.int64)
    pl = np.ascontiguousarray([x[1] for x in arrivals], dtype=np.int32)
    ol = np.ascontiguousarray([x[2] for x in arrivals], dtype=np.int32)
    cp, cm, res = params.c(), gllm_stage_time_model(*model), gllm_sim_result()
    if len(arrivals) and len(arrivals[0]) > 3:
        tk = np.ascontiguousarray(np.concatenate([np.asarray(x[3], dtype=np.int32) for x in arrivals]))
        if len(tk) != int(pl.sum()):
            raise ValueError("each prompt must come with prompt_len token ids")
        st = _lib().gllm_sched_simulate_tokens(C.byref(cp), C.byref(cm), _ptr(a, C.c_int64), _ptr(pl, C.c_int32),
                                               _ptr(ol, C.c_int32), _ptr(tk, C.c_int32), len(a), C.byref(res))
    else:
        st = _lib().gllm_sched_simulate(C.byref(cp), C.byref(cm), _ptr(a, C.c_int64), _ptr(pl, C.c_int32), _ptr(ol, C.c_int32),
                                        len(a), C.byref(res))
    if st != GLLM_OK:
        raise GllmError(st, "gllm_sched_simulate")
    return {n: int(getattr(res, n)) for n in SIM_FIELDS}
