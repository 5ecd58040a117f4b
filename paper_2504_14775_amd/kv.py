"""ctypes binding of the KV page pool (include/gllm_kv.h): argument marshalling only."""
from __future__ import annotations

import ctypes as C
from typing import List

import numpy as np

from .binding import GLLM_OK, GllmError, load_host_library

EXPORTS = [
    "gllm_kv_create", "gllm_kv_destroy", "gllm_kv_available", "gllm_kv_alloc", "gllm_kv_match", "gllm_kv_register",
    "gllm_kv_release", "gllm_kv_get_state", "gllm_kv_page_info",
]

PAGE_TOKENS, ROOT = 16, -1


class gllm_kv_state(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("total_pages", "free_pages", "idle_cached_pages", "registered_pages", "evictions")]


_ready = False


def _lib():
    global _ready
    lib = load_host_library()
    if not _ready:
        i32, i64, vp = C.c_int32, C.c_int64, C.c_void_p
        P = C.POINTER
        lib.gllm_kv_create.restype = i32
        lib.gllm_kv_create.argtypes = [i64, P(vp)]
        lib.gllm_kv_destroy.restype = None
        lib.gllm_kv_destroy.argtypes = [vp]
        lib.gllm_kv_available.restype = i64
        lib.gllm_kv_available.argtypes = [vp]
        lib.gllm_kv_alloc.restype = i32
        lib.gllm_kv_alloc.argtypes = [vp, i32, P(i32)]
        lib.gllm_kv_match.restype = i32
        lib.gllm_kv_match.argtypes = [vp, P(i32), i64, i32, P(i32), P(i32)]
        lib.gllm_kv_register.restype = i32
        lib.gllm_kv_register.argtypes = [vp, i32, P(i32), i32, P(i32)]
        lib.gllm_kv_release.restype = i32
        lib.gllm_kv_release.argtypes = [vp, P(i32), i32]
        lib.gllm_kv_get_state.restype = i32
        lib.gllm_kv_get_state.argtypes = [vp, P(gllm_kv_state)]
        lib.gllm_kv_page_info.restype = i32
        lib.gllm_kv_page_info.argtypes = [vp, i32, P(i32), P(i32), P(i32)]
        _ready = True
    return lib


def _i32(values) -> np.ndarray:
    return np.ascontiguousarray(values, dtype=np.int32)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


class PagePool:
    def __init__(self, total_pages: int):
        self.lib = _lib()
        h = C.c_void_p()
        st = self.lib.gllm_kv_create(total_pages, C.byref(h))
        if st != GLLM_OK:
            raise GllmError(st, "gllm_kv_create")
        self.handle = h

    def __del__(self):
        if getattr(self, "handle", None):
            self.lib.gllm_kv_destroy(self.handle)
            self.handle = None

    def _check(self, st: int, what: str) -> None:
        if st != GLLM_OK:
            raise GllmError(st, what)

    def available(self) -> int:
        return int(self.lib.gllm_kv_available(self.handle))

    def alloc(self, n: int = 1) -> List[int]:
        out = np.empty(max(n, 1), dtype=np.int32)
        self._check(self.lib.gllm_kv_alloc(self.handle, n, _ptr(out)), "gllm_kv_alloc")
        return [int(x) for x in out[:n]]

    def match(self, tokens, max_pages: int) -> List[int]:
        t = _i32(tokens)
        out = np.empty(max(max_pages, 1), dtype=np.int32)
        n = C.c_int32(0)
        self._check(self.lib.gllm_kv_match(self.handle, _ptr(t), len(t), max_pages, _ptr(out), C.byref(n)), "gllm_kv_match")
        return [int(x) for x in out[:n.value]]

    def register(self, parent: int, tokens16, page: int) -> bool:
        t = _i32(tokens16)
        if t.shape != (PAGE_TOKENS,):
            raise ValueError("a page holds 16 token ids")
        ok = C.c_int32(0)
        self._check(self.lib.gllm_kv_register(self.handle, parent, _ptr(t), page, C.byref(ok)), "gllm_kv_register")
        return bool(ok.value)

    def release(self, pages) -> None:
        t = _i32(pages)
        self._check(self.lib.gllm_kv_release(self.handle, _ptr(t), len(t)), "gllm_kv_release")

    def state(self) -> dict:
        st = gllm_kv_state()
        self._check(self.lib.gllm_kv_get_state(self.handle, C.byref(st)), "gllm_kv_get_state")
        return {n: int(getattr(st, n)) for n, _ in gllm_kv_state._fields_}

    def page_info(self, page: int) -> tuple:
        h, r, c = C.c_int32(0), C.c_int32(0), C.c_int32(0)
        self._check(self.lib.gllm_kv_page_info(self.handle, page, C.byref(h), C.byref(r), C.byref(c)), "gllm_kv_page_info")
        return int(h.value), bool(r.value), int(c.value)
