"""CPU oracle: build helper and numpy/ctypes wrapper.  TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package.
It imports nothing from the HIP library.  All arithmetic lives in stage_oracle.c; this file
only marshals numpy arrays (bf16 travels as uint16 bit patterns, everything else as float64
or int32).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "stage_oracle.c")
_SO = os.path.join(_HERE, "libstage_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile stage_oracle.c with gcc (baseline x86-64 plus runtime-dispatched clones)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        # -ffp-contract=off: no fused multiply-add, every operation rounds on its own, so results do not
        # depend on the instruction set of the host or on the loop nest that produced them
        cmd = ["gcc", "-O2", "-ftree-vectorize", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
               "-std=gnu11", "-Wall", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


class Config(C.Structure):
    _fields_ = [("num_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("intermediate", C.c_int32),
                ("page_size", C.c_int32), ("has_qkv_bias", C.c_int32),
                ("rms_eps", C.c_double), ("rope_theta", C.c_double),
                ("round_operands", C.c_int32), ("reserved", C.c_int32)]


_W_FIELDS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "norm1", "norm2", "bq", "bk", "bv")


class Layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _W_FIELDS]


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = C.CDLL(_SO)
        _lib.oracle_bf16_to_f64.restype = C.c_double
        _lib.oracle_bf16_to_f64.argtypes = [C.c_uint16]
        _lib.oracle_f64_to_bf16.restype = C.c_uint16
        _lib.oracle_f64_to_bf16.argtypes = [C.c_double]
        _lib.oracle_k_index.restype = C.c_int64
        _lib.oracle_v_index.restype = C.c_int64
        for f in (_lib.oracle_k_index, _lib.oracle_v_index):
            f.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int64, C.c_int, C.c_int, C.c_int]
        _lib.oracle_token_map.restype = C.c_int64
        _lib.oracle_stage_forward.restype = C.c_int
        _lib.oracle_layer_rows.restype = C.c_int
    return _lib


def make_config(shape, round_operands: bool = False) -> Config:
    """shape: any object with the StageShape attribute names."""
    return Config(shape.num_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                  shape.intermediate, shape.page_size, int(bool(shape.has_qkv_bias)),
                  float(shape.rms_eps), float(shape.rope_theta), int(bool(round_operands)), 0)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (pure bit placement, no arithmetic)."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f64_to_bf16(x: np.ndarray) -> np.ndarray:
    x = _f64(x)
    L = lib()
    out = np.empty(x.shape, dtype=np.uint16)
    L.oracle_f64_to_bf16_array(C.c_int64(x.size), _p(x), _p(out))
    return out


def make_layer(weights: Dict[str, np.ndarray]) -> Layer:
    """weights: name -> uint16 array (bf16 bits).  The caller keeps the arrays alive."""
    lay = Layer()
    for n in _W_FIELDS:
        a = weights.get(n)
        if a is not None:
            assert a.dtype == np.uint16 and a.flags.c_contiguous, n
        setattr(lay, n, None if a is None else a.ctypes.data)
    return lay


def token_map(new_tokens, cached_len):
    nt, cl = _i32(new_tokens), _i32(cached_len)
    T = int(nt.sum())
    seq_of = np.empty(T, dtype=np.int32)
    pos_of = np.empty(T, dtype=np.int32)
    lib().oracle_token_map(C.c_int(len(nt)), _p(nt), _p(cl), _p(seq_of), _p(pos_of))
    return seq_of, pos_of


def rmsnorm(x, gamma_bits, eps: float) -> np.ndarray:
    x = _f64(x)
    T, H = x.shape
    out = np.empty_like(x)
    lib().oracle_rmsnorm(C.c_int64(T), C.c_int(H), _p(x), _p(_u16(gamma_bits)), C.c_double(eps), _p(out))
    return out


def linear(x, w_bits, bias_bits=None) -> np.ndarray:
    x = _f64(x)
    w = _u16(w_bits)
    T, K = x.shape
    N = w.shape[0]
    assert w.shape[1] == K
    y = np.empty((T, N), dtype=np.float64)
    b = None if bias_bits is None else _u16(bias_bits)
    lib().oracle_linear(C.c_int64(T), C.c_int(K), C.c_int(N), _p(x), _p(w), _p(b), _p(y))
    return y


def rope(v, pos, base: float) -> np.ndarray:
    """v: [T, n_heads, d] -> rotated copy."""
    v = _f64(v).copy()
    T, nh, d = v.shape
    lib().oracle_rope(C.c_int64(T), C.c_int(nh), C.c_int(d), _p(_i32(pos)), C.c_double(base), _p(v))
    return v


def swiglu(gate, up) -> np.ndarray:
    g, u = _f64(gate), _f64(up)
    a = np.empty_like(g)
    lib().oracle_swiglu(C.c_int64(g.size), _p(g), _p(u), _p(a))
    return a


def kv_write(shape, layer, seq_of, pos_of, block_tables, num_pages, k, v, k_pool, v_pool) -> None:
    cfg = make_config(shape)
    bt = _i32(block_tables)
    k, v = _f64(k), _f64(v)
    lib().oracle_kv_write(C.byref(cfg), C.c_int(layer), C.c_int64(len(seq_of)), _p(_i32(seq_of)),
                          _p(_i32(pos_of)), _p(bt), C.c_int(bt.shape[1]), C.c_int64(num_pages),
                          _p(k), _p(v), _p(_u16(k_pool)), _p(_u16(v_pool)))


def attention(shape, layer, seq_of, pos_of, block_tables, num_pages, q, k_pool, v_pool) -> np.ndarray:
    """q: [T, n_q, d] float64 -> o: [T, n_q, d] float64."""
    cfg = make_config(shape)
    bt = _i32(block_tables)
    q = _f64(q)
    o = np.empty_like(q)
    lib().oracle_attention(C.byref(cfg), C.c_int(layer), C.c_int64(len(seq_of)), _p(_i32(seq_of)),
                           _p(_i32(pos_of)), _p(bt), C.c_int(bt.shape[1]), C.c_int64(num_pages),
                           _p(q), _p(_u16(k_pool)), _p(_u16(v_pool)), _p(o))
    return o


def layer_forward(shape, layer: int, weights: Dict[str, np.ndarray], seq_of, pos_of, block_tables,
                  num_pages: int, k_pool: np.ndarray, v_pool: np.ndarray, x: np.ndarray):
    """One decoder layer on the residual stream x [T,H] float64 (copied).

    Returns (x_after_layer, x_after_attention_half); pools are updated in place.
    """
    cfg = make_config(shape)
    lay = make_layer(weights)
    bt = _i32(block_tables)
    x = _f64(x).copy()
    tap = np.empty_like(x)
    lib().oracle_layer_forward(C.byref(cfg), C.c_int(layer), C.byref(lay), C.c_int64(x.shape[0]),
                               _p(_i32(seq_of)), _p(_i32(pos_of)), _p(bt), C.c_int(bt.shape[1]),
                               C.c_int64(num_pages), _p(k_pool), _p(v_pool), _p(x), _p(tap))
    return x, tap


def pool_index(shape, which: str, num_pages: int, layer: int, page: int, kvh: int, slot: int, dim: int) -> int:
    cfg = make_config(shape)
    f = lib().oracle_k_index if which == "k" else lib().oracle_v_index
    return int(f(C.byref(cfg), num_pages, layer, page, kvh, slot, dim))


def stage_forward(shape, layers: Sequence[Dict[str, np.ndarray]], new_tokens, cached_len, block_tables,
                  num_pages: int, k_pool: np.ndarray, v_pool: np.ndarray, hidden_bits: np.ndarray,
                  round_operands: bool = False):
    """Runs the stage; k_pool / v_pool (uint16, flat) are updated in place.

    round_operands selects the diagnostic reading (bf16 tensors in front of every matrix product).
    Returns (out_f64 [T,H], out_bf16_bits [T,H]).
    """
    cfg = make_config(shape, round_operands)
    arr = (Layer * len(layers))(*[make_layer(w) for w in layers])
    nt, cl, bt = _i32(new_tokens), _i32(cached_len), _i32(block_tables)
    T = int(nt.sum())
    hid = _u16(hidden_bits)
    assert hid.shape == (T, shape.hidden)
    assert k_pool.dtype == np.uint16 and v_pool.dtype == np.uint16
    assert k_pool.flags.c_contiguous and v_pool.flags.c_contiguous
    out = np.empty((T, shape.hidden), dtype=np.float64)
    outb = np.empty((T, shape.hidden), dtype=np.uint16)
    rc = lib().oracle_stage_forward(C.byref(cfg), arr, C.c_int(len(nt)), _p(nt), _p(cl), _p(bt),
                                    C.c_int(bt.shape[1]), C.c_int64(num_pages), _p(k_pool), _p(v_pool),
                                    _p(hid), _p(out), _p(outb))
    if rc != 0:
        raise ValueError(f"oracle_stage_forward rejected the batch (rc={rc})")
    return out, outb


def layer_rows(shape, layer: int, weights: Dict[str, np.ndarray], new_tokens, cached_len, block_tables,
               num_pages: int, k_pool: np.ndarray, v_pool: np.ndarray, hidden_bits: np.ndarray,
               need: Optional[np.ndarray] = None, round_operands: bool = False) -> np.ndarray:
    """Layer `layer` of the stage alone (its weights, its slice of the pools, which hold all layers of `shape`).

    hidden_bits [T,H] is the residual stream in front of the layer (bf16 bits); need [T] (bool, None = all) selects
    the rows that are carried through the layer; every row writes its K and V into the pools (updated in place).
    Returns out_f64 [T,H]: the stream behind the layer on the needed rows, the widened input elsewhere.
    """
    cfg = make_config(shape, round_operands)
    lay = make_layer(weights)
    nt, cl, bt = _i32(new_tokens), _i32(cached_len), _i32(block_tables)
    T = int(nt.sum())
    hid = _u16(hidden_bits)
    assert hid.shape == (T, shape.hidden)
    assert k_pool.dtype == np.uint16 and v_pool.dtype == np.uint16
    assert k_pool.flags.c_contiguous and v_pool.flags.c_contiguous
    nd = None
    if need is not None:
        nd = np.ascontiguousarray(need, dtype=np.uint8)
        assert nd.shape == (T,)
    out = np.empty((T, shape.hidden), dtype=np.float64)
    rc = lib().oracle_layer_rows(C.byref(cfg), C.c_int(layer), C.byref(lay), C.c_int(len(nt)), _p(nt), _p(cl), _p(bt),
                                 C.c_int(bt.shape[1]), C.c_int64(num_pages), _p(k_pool), _p(v_pool), _p(hid),
                                 _p(nd), _p(out))
    if rc != 0:
        raise ValueError(f"oracle_layer_rows rejected the batch (rc={rc})")
    return out
