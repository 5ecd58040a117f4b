"""Thin ctypes binding of libgllm_stage.so (declared in include/gllm_stage.h).

Argument marshalling only: every step of the stage runs in the library's HIP kernels.  PyTorch
is used for device memory (torch tensors -> data_ptr()) and streams, nothing else.  If the
library is missing or cannot be loaded this module raises; there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgllm_stage.so")

GLLM_OK = 0
STATUS = {0: "GLLM_OK", -1: "GLLM_E_INVALID", -2: "GLLM_E_CAPACITY", -3: "GLLM_E_BLOCK_RANGE",
          -4: "GLLM_E_BLOCK_ALIAS", -5: "GLLM_E_STATE", -6: "GLLM_E_HIP", -7: "GLLM_E_UNSUPPORTED"}
GEMM_STORE_F32, GEMM_ADD_F32, GEMM_SWIGLU_BF16 = 0, 1, 2

EXPORTS = [
    "gllm_stage_create", "gllm_stage_destroy", "gllm_last_error", "gllm_status_name",
    "gllm_stage_workspace_bytes", "gllm_stage_bind_workspace", "gllm_stage_load_layer",
    "gllm_stage_bind_kv_pool", "gllm_stage_share_weights", "gllm_stage_set_alias_check", "gllm_stage_set_option", "gllm_stage_forward",
    "gllm_stage_set_profiling", "gllm_stage_read_profile", "gllm_profile_num_classes",
    "gllm_profile_class_name", "gllm_op_pack_weight", "gllm_op_gemm_bf16", "gllm_op_gemm_bf16_splitk", "gllm_op_gemm_plan", "gllm_op_rmsnorm", "gllm_op_peak_mfma", "gllm_op_peak_read", "gllm_op_peak_read_nt",
]


class GllmError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status
        self.message = message


class gllm_stage_config(C.Structure):
    _fields_ = [("num_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("intermediate", C.c_int32),
                ("page_size", C.c_int32), ("has_qkv_bias", C.c_int32), ("max_tokens", C.c_int32),
                ("max_seqs", C.c_int32), ("max_blocks_per_seq", C.c_int32), ("max_position", C.c_int32),
                ("rms_eps", C.c_double), ("rope_theta", C.c_double)]


_W_FIELDS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "norm1", "norm2", "bq", "bk", "bv")


class gllm_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _W_FIELDS]


class gllm_batch(C.Structure):
    _fields_ = [("num_seqs", C.c_int32), ("block_table_stride", C.c_int32),
                ("new_tokens", C.POINTER(C.c_int32)), ("cached_len", C.POINTER(C.c_int32)),
                ("block_tables", C.POINTER(C.c_int32))]


_lib = None
_host_lib = None


def load_host_library():
    """The library that holds the host-only entry points (scheduler, KV page pool).

    Normally that is libgllm_stage.so itself.  GLLM_HOST_LIBRARY may name another build of the two host sources
    (csrc/gllm_sched.cpp, csrc/gllm_kv.cpp) instead -- the sanitizer build of build.build_host_sanitized(), which
    the CPU tests run the parity suites against; such a library is loaded without touching torch or HIP."""
    global _host_lib
    if _host_lib is None:
        path = os.environ.get("GLLM_HOST_LIBRARY")
        _host_lib = C.CDLL(path) if path else load_library()
    return _host_lib


def load_library():
    """Loads the shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    # torch first: the library must bind to the HIP runtime that torch has loaded, so that device
    # pointers and streams handed over from torch tensors belong to the same runtime instance
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2504_14775_amd.build` "
                          "(there is no fallback implementation)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.gllm_stage_create.restype = i32
    lib.gllm_stage_create.argtypes = [C.POINTER(gllm_stage_config), C.POINTER(vp)]
    lib.gllm_stage_destroy.restype = None
    lib.gllm_stage_destroy.argtypes = [vp]
    lib.gllm_last_error.restype = C.c_char_p
    lib.gllm_last_error.argtypes = [vp]
    lib.gllm_status_name.restype = C.c_char_p
    lib.gllm_status_name.argtypes = [i32]
    lib.gllm_stage_workspace_bytes.restype = C.c_size_t
    lib.gllm_stage_workspace_bytes.argtypes = [vp]
    lib.gllm_stage_bind_workspace.restype = i32
    lib.gllm_stage_bind_workspace.argtypes = [vp, vp, C.c_size_t]
    lib.gllm_stage_load_layer.restype = i32
    lib.gllm_stage_load_layer.argtypes = [vp, i32, C.POINTER(gllm_layer_weights), vp]
    lib.gllm_stage_bind_kv_pool.restype = i32
    lib.gllm_stage_bind_kv_pool.argtypes = [vp, vp, vp, i64]
    lib.gllm_stage_set_alias_check.restype = i32
    lib.gllm_stage_set_alias_check.argtypes = [vp, i32]
    lib.gllm_stage_share_weights.restype = i32
    lib.gllm_stage_share_weights.argtypes = [vp, vp]
    lib.gllm_stage_set_option.restype = i32
    lib.gllm_stage_set_option.argtypes = [vp, C.c_char_p, i64]
    lib.gllm_stage_forward.restype = i32
    lib.gllm_stage_forward.argtypes = [vp, C.POINTER(gllm_batch), vp, vp, vp, vp]
    lib.gllm_stage_set_profiling.restype = i32
    lib.gllm_stage_set_profiling.argtypes = [vp, i32]
    lib.gllm_stage_read_profile.restype = i32
    lib.gllm_stage_read_profile.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64), i32]
    lib.gllm_profile_num_classes.restype = i32
    lib.gllm_profile_num_classes.argtypes = []
    lib.gllm_profile_class_name.restype = C.c_char_p
    lib.gllm_profile_class_name.argtypes = [i32]
    lib.gllm_op_pack_weight.restype = i32
    lib.gllm_op_pack_weight.argtypes = [vp, i64, i32, i32, vp, vp]
    lib.gllm_op_gemm_bf16.restype = i32
    lib.gllm_op_gemm_bf16.argtypes = [vp, i64, vp, i64, vp, i64, i32, i32, i32, i32, i32, vp]
    lib.gllm_op_gemm_bf16_splitk.restype = i32
    lib.gllm_op_gemm_bf16_splitk.argtypes = [vp, i64, vp, i64, vp, i64, i32, i32, i32, i32, i32, i64, vp]
    lib.gllm_op_gemm_plan.restype = i32
    lib.gllm_op_gemm_plan.argtypes = [i32, i32, i32, i32, i32, C.POINTER(i32), C.POINTER(i32)]
    lib.gllm_op_rmsnorm.restype = i32
    lib.gllm_op_rmsnorm.argtypes = [vp, vp, vp, i32, i32, C.c_double, vp]
    lib.gllm_op_peak_mfma.restype = i32
    lib.gllm_op_peak_mfma.argtypes = [vp, i32, i32, vp]
    lib.gllm_op_peak_read.restype = i32
    lib.gllm_op_peak_read.argtypes = [vp, i64, vp, i32, vp]
    lib.gllm_op_peak_read_nt.restype = i32
    lib.gllm_op_peak_read_nt.argtypes = [vp, i64, vp, i32, vp]
    _lib = lib
    return lib


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def make_config(shape, max_tokens: int, max_seqs: int, max_blocks_per_seq: int, max_position: int) -> gllm_stage_config:
    return gllm_stage_config(shape.num_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                             shape.intermediate, shape.page_size, int(bool(shape.has_qkv_bias)), max_tokens,
                             max_seqs, max_blocks_per_seq, max_position, float(shape.rms_eps),
                             float(shape.rope_theta))


class Stage:
    """Owner of one gllm_stage handle.  Methods carry the names of the C entry points."""

    def __init__(self, cfg: gllm_stage_config):
        self.lib = load_library()
        self.cfg = cfg
        handle = C.c_void_p()
        st = self.lib.gllm_stage_create(C.byref(cfg), C.byref(handle))
        if st != GLLM_OK:
            raise GllmError(st, self.lib.gllm_last_error(None).decode())
        self.handle = handle
        self._keep = []

    def _check(self, st: int):
        if st != GLLM_OK:
            raise GllmError(st, self.lib.gllm_last_error(self.handle).decode())

    def destroy(self):
        if getattr(self, "handle", None):
            self.lib.gllm_stage_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def workspace_bytes(self) -> int:
        return int(self.lib.gllm_stage_workspace_bytes(self.handle))

    def bind_workspace(self, tensor) -> None:
        self._check(self.lib.gllm_stage_bind_workspace(self.handle, tensor.data_ptr(), tensor.numel() * tensor.element_size()))
        self._keep.append(tensor)

    def load_layer(self, layer: int, weights: Dict[str, "object"], stream=None) -> None:
        w = gllm_layer_weights()
        for n in _W_FIELDS:
            t = weights.get(n)
            setattr(w, n, None if t is None else t.data_ptr())
        self._check(self.lib.gllm_stage_load_layer(self.handle, layer, C.byref(w), _stream_ptr(stream)))

    def bind_kv_pool(self, k_pool, v_pool, num_blocks: int) -> None:
        self._check(self.lib.gllm_stage_bind_kv_pool(self.handle, k_pool.data_ptr(), v_pool.data_ptr(), num_blocks))
        self._pool = (k_pool, v_pool)

    def share_weights(self, owner: "Stage") -> None:
        """Use owner's loaded weights instead of a copy of one's own (owner must outlive this stage)."""
        self._check(self.lib.gllm_stage_share_weights(self.handle, owner.handle))
        self._owner = owner

    def set_alias_check(self, on: bool) -> None:
        self._check(self.lib.gllm_stage_set_alias_check(self.handle, int(on)))

    def set_option(self, name: str, value: int) -> None:
        self._check(self.lib.gllm_stage_set_option(self.handle, name.encode(), int(value)))

    def forward(self, new_tokens, cached_len, block_tables, hidden_in, hidden_out, hidden_out_f32=None,
                stream=None) -> None:
        nt = np.ascontiguousarray(new_tokens, dtype=np.int32)
        cl = np.ascontiguousarray(cached_len, dtype=np.int32)
        bt = np.ascontiguousarray(block_tables, dtype=np.int32)
        assert bt.ndim == 2 and bt.shape[0] == nt.shape[0] == cl.shape[0]
        ip = C.POINTER(C.c_int32)
        b = gllm_batch(int(nt.shape[0]), int(bt.shape[1]), nt.ctypes.data_as(ip), cl.ctypes.data_as(ip),
                       bt.ctypes.data_as(ip))
        f32 = None if hidden_out_f32 is None else hidden_out_f32.data_ptr()
        self._check(self.lib.gllm_stage_forward(self.handle, C.byref(b), hidden_in.data_ptr(), hidden_out.data_ptr(),
                                                f32, _stream_ptr(stream)))

    def forward_raw(self, batch: gllm_batch, hidden_in_ptr, hidden_out_ptr, hidden_out_f32_ptr, stream_ptr) -> int:
        """Unchecked call (returns the status), for tests of the error paths."""
        return self.lib.gllm_stage_forward(self.handle, C.byref(batch) if batch is not None else None, hidden_in_ptr,
                                           hidden_out_ptr, hidden_out_f32_ptr, stream_ptr)

    def last_error(self) -> str:
        return self.lib.gllm_last_error(self.handle).decode()

    def set_profiling(self, on: bool) -> None:
        self._check(self.lib.gllm_stage_set_profiling(self.handle, int(on)))

    def read_profile(self, reset: bool = True) -> Dict[str, Tuple[float, int]]:
        n = self.lib.gllm_profile_num_classes()
        ms = (C.c_double * n)()
        cnt = (C.c_int64 * n)()
        self._check(self.lib.gllm_stage_read_profile(self.handle, ms, cnt, int(reset)))
        return {self.lib.gllm_profile_class_name(i).decode(): (float(ms[i]), int(cnt[i])) for i in range(n)}


def gllm_op_pack_weight(w, out, stream=None):
    """w: bf16 [n, k] row-major (device); out: bf16, n*k elements, receives the GEMM's tiled weight layout."""
    lib = load_library()
    st = lib.gllm_op_pack_weight(w.data_ptr(), w.stride(0), w.shape[0], w.shape[1], out.data_ptr(), _stream_ptr(stream))
    if st != GLLM_OK:
        raise GllmError(st, "gllm_op_pack_weight")


def gllm_op_gemm_bf16(a, w, out, m: int, n: int, k: int, mode: int, tile: int = -1, lda=None, ldw=None, ldc=None,
                      stream=None):
    """w: a [n, k] tensor holding the tiled layout gllm_op_pack_weight writes (its row stride is taken as the k extent)."""
    lib = load_library()
    st = lib.gllm_op_gemm_bf16(a.data_ptr(), lda or a.stride(0), w.data_ptr(), ldw or w.stride(0), out.data_ptr(),
                               ldc or out.stride(0), m, n, k, mode, tile, _stream_ptr(stream))
    if st != GLLM_OK:
        raise GllmError(st, "gllm_op_gemm_bf16")


def gllm_op_gemm_bf16_splitk(a, w, out_planes, m: int, n: int, k: int, tile: int, splits: int, stream=None):
    """out_planes: fp32 [splits, m, n]."""
    lib = load_library()
    st = lib.gllm_op_gemm_bf16_splitk(a.data_ptr(), a.stride(0), w.data_ptr(), w.stride(0), out_planes.data_ptr(),
                                      out_planes.stride(1), m, n, k, tile, splits, out_planes.stride(0),
                                      _stream_ptr(stream))
    if st != GLLM_OK:
        raise GllmError(st, "gllm_op_gemm_bf16_splitk")


def gllm_op_gemm_plan(m: int, n: int, k: int, mode: int, max_splits: int):
    """(tile, splits) the library would use for this problem; host only."""
    lib = load_library()
    tile, splits = C.c_int32(-1), C.c_int32(0)
    st = lib.gllm_op_gemm_plan(m, n, k, mode, max_splits, C.byref(tile), C.byref(splits))
    if st != GLLM_OK:
        raise GllmError(st, "gllm_op_gemm_plan")
    return tile.value, splits.value


def gllm_op_rmsnorm(x, gamma, h, eps: float, stream=None):
    lib = load_library()
    st = lib.gllm_op_rmsnorm(x.data_ptr(), gamma.data_ptr(), h.data_ptr(), x.shape[0], x.shape[1], eps,
                             _stream_ptr(stream))
    if st != GLLM_OK:
        raise GllmError(st, "gllm_op_rmsnorm")


def gllm_op_peak_mfma(sink, workgroups: int, iters: int, stream=None):
    st = load_library().gllm_op_peak_mfma(sink.data_ptr(), workgroups, iters, _stream_ptr(stream))
    if st != GLLM_OK:
        raise GllmError(st, "gllm_op_peak_mfma")


def gllm_op_peak_read(src, nbytes: int, sink, workgroups: int, stream=None, non_temporal: bool = False):
    lib = load_library()
    fn = lib.gllm_op_peak_read_nt if non_temporal else lib.gllm_op_peak_read
    st = fn(src.data_ptr(), nbytes, sink.data_ptr(), workgroups, _stream_ptr(stream))
    if st != GLLM_OK:
        raise GllmError(st, "gllm_op_peak_read")


def stage_for_batches(shape, batches: Sequence, device="cuda"):
    """Creates a Stage sized for the given batches, with its workspace bound (torch allocates)."""
    import torch
    max_tokens = max(b.num_tokens for b in batches)
    max_seqs = max(b.num_seqs for b in batches)
    max_pos = max(int((b.new_tokens + b.cached_len).max()) for b in batches)
    max_blocks = max(b.block_tables.shape[1] for b in batches)
    max_blocks = max(max_blocks, (max_pos + shape.page_size - 1) // shape.page_size)
    st = Stage(make_config(shape, max_tokens, max_seqs, max_blocks, max_pos))
    ws = torch.empty(st.workspace_bytes(), dtype=torch.uint8, device=device)
    st.bind_workspace(ws)
    return st
