"""ctypes binding of the first / last stage extras (include/gllm_head.h): argument marshalling only."""
from __future__ import annotations

import ctypes as C

from .binding import GLLM_OK, GllmError, _stream_ptr, load_library

EXPORTS = [
    "gllm_op_embedding", "gllm_head_create", "gllm_head_destroy", "gllm_head_last_error", "gllm_head_workspace_bytes",
    "gllm_head_bind_workspace", "gllm_head_load", "gllm_head_logits", "gllm_head_padded_vocab", "gllm_op_sample",
    "gllm_head_logits_static", "gllm_head_static_scratch_bytes",
]


class gllm_head_config(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("vocab", C.c_int32), ("max_rows", C.c_int32), ("reserved", C.c_int32),
                ("rms_eps", C.c_double)]


_ready = False


def _lib():
    global _ready
    lib = load_library()
    if not _ready:
        i32, i64, vp = C.c_int32, C.c_int64, C.c_void_p
        lib.gllm_op_embedding.restype = i32
        lib.gllm_op_embedding.argtypes = [vp, vp, vp, i32, i32, i32, i64, vp]
        lib.gllm_head_create.restype = i32
        lib.gllm_head_create.argtypes = [C.POINTER(gllm_head_config), C.POINTER(vp)]
        lib.gllm_head_destroy.restype = None
        lib.gllm_head_destroy.argtypes = [vp]
        lib.gllm_head_last_error.restype = C.c_char_p
        lib.gllm_head_last_error.argtypes = [vp]
        lib.gllm_head_workspace_bytes.restype = C.c_size_t
        lib.gllm_head_workspace_bytes.argtypes = [vp]
        lib.gllm_head_bind_workspace.restype = i32
        lib.gllm_head_bind_workspace.argtypes = [vp, vp, C.c_size_t]
        lib.gllm_head_load.restype = i32
        lib.gllm_head_load.argtypes = [vp, vp, vp, vp]
        lib.gllm_head_logits.restype = i32
        lib.gllm_head_logits.argtypes = [vp, vp, i32, vp, i32, vp, i64, vp]
        lib.gllm_head_logits_static.restype = i32
        lib.gllm_head_logits_static.argtypes = [vp, vp, i32, vp, i32, vp, i64, vp]
        lib.gllm_head_static_scratch_bytes.restype = C.c_size_t
        lib.gllm_head_static_scratch_bytes.argtypes = []
        lib.gllm_head_padded_vocab.restype = i32
        lib.gllm_head_padded_vocab.argtypes = [vp]
        lib.gllm_op_sample.restype = i32
        lib.gllm_op_sample.argtypes = [vp, i64, i32, i32, vp, vp, vp, vp, vp, vp]
        _ready = True
    return lib


def gllm_op_embedding(ids, table, out, stream=None) -> None:
    """ids: int32 [T] (device), table: bf16 [V, H], out: bf16 [T, >=H] (row stride taken from the tensor)."""
    st = _lib().gllm_op_embedding(ids.data_ptr(), table.data_ptr(), out.data_ptr(), ids.shape[0], table.shape[1],
                                  table.shape[0], out.stride(0), _stream_ptr(stream))
    if st != GLLM_OK:
        raise GllmError(st, "gllm_op_embedding")


def gllm_op_sample(logits, vocab: int, temperature, top_k, top_p, u, out_ids, stream=None) -> None:
    st = _lib().gllm_op_sample(logits.data_ptr(), logits.stride(0), logits.shape[0], vocab, temperature.data_ptr(),
                               top_k.data_ptr(), top_p.data_ptr(), u.data_ptr(), out_ids.data_ptr(), _stream_ptr(stream))
    if st != GLLM_OK:
        raise GllmError(st, "gllm_op_sample")


class Head:
    def __init__(self, hidden: int, vocab: int, max_rows: int, rms_eps: float, device="cuda", bind_workspace: bool = True):
        import torch
        self.lib = _lib()
        cfg = gllm_head_config(hidden, vocab, max_rows, 0, rms_eps)
        h = C.c_void_p()
        st = self.lib.gllm_head_create(C.byref(cfg), C.byref(h))
        if st != GLLM_OK:
            raise GllmError(st, "gllm_head_create")
        self.handle = h
        self.vocab = vocab
        self.padded_vocab = int(self.lib.gllm_head_padded_vocab(h))
        if bind_workspace:
            self._ws = torch.empty(int(self.lib.gllm_head_workspace_bytes(h)), dtype=torch.uint8, device=device)
            self._check(self.lib.gllm_head_bind_workspace(h, self._ws.data_ptr(), self._ws.numel()))

    def _check(self, st: int) -> None:
        if st != GLLM_OK:
            raise GllmError(st, self.lib.gllm_head_last_error(self.handle).decode())

    def destroy(self) -> None:
        if getattr(self, "handle", None):
            self.lib.gllm_head_destroy(self.handle)
            self.handle = None

    def __del__(self):
        self.destroy()

    def load(self, norm_gain, w_vocab, stream=None) -> None:
        self._check(self.lib.gllm_head_load(self.handle, norm_gain.data_ptr(), w_vocab.data_ptr(), _stream_ptr(stream)))

    def logits(self, x, rows, out, stream=None) -> None:
        """x: fp32 [T, H]; rows: int32 [M] (device); out: fp32 [M, >= padded_vocab]."""
        self._check(self.lib.gllm_head_logits(self.handle, x.data_ptr(), x.shape[0], rows.data_ptr(), rows.shape[0],
                                              out.data_ptr(), out.stride(0), _stream_ptr(stream)))

    def logits_static(self, x, rows, out, stream=None) -> None:
        """The same through gllm_head_logits_static (scratch inside the library, no workspace needed)."""
        self._check(self.lib.gllm_head_logits_static(self.handle, x.data_ptr(), x.shape[0], rows.data_ptr(), rows.shape[0],
                                                     out.data_ptr(), out.stride(0), _stream_ptr(stream)))
