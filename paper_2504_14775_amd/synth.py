"""Seeded synthetic inputs for one pipeline stage's forward pass.

This module only *generates data*: stage shapes, layer weights, hidden inputs,
paged-KV pool contents, block tables and batch descriptors.  It contains none of
the stage's arithmetic (no norm, GEMM, RoPE, attention), and it imports neither
the CPU oracle nor the HIP library; both are fed the buffers produced here.

The batches follow the workload structure of the paper: hybrid micro-batches of
chunked-prefill tokens and single-token decode rows under a 2048-token budget
(paper section 2.2, "Scheduling Policies", and section 4.1, token budget), paged
KV with per-sequence page tables shared by every stage (section 3.3), bf16 data
(section 4.1), and a PP=4 stage's share of the layers of Llama/Qwen-shaped models.
The paper's request traces are not used; sequence lengths are drawn from the
stated distributions instead.

Randomness is counter based: value = f(seed, stream, element index), so any slice
of any tensor can be produced on any device in any order.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import numpy as np
import torch

PAGE = 16  # tokens per KV page (all configurations)

# ----------------------------------------------------------------------------
# counter-based generator
# ----------------------------------------------------------------------------
_M64 = (1 << 64) - 1


def _as_i64(v: int) -> int:
    """Two's-complement view of a 64-bit unsigned constant (torch has no uint64 math)."""
    v &= _M64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = _as_i64(0x9E3779B97F4A7C15)
_MUL1 = _as_i64(0xBF58476D1CE4E5B9)
_MUL2 = _as_i64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 lanes."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(z: torch.Tensor) -> torch.Tensor:
    """64-bit avalanche finaliser (two xor-shift-multiply rounds and a last xor-shift)."""
    z = (z ^ _lsr(z, 30)) * _MUL1
    z = (z ^ _lsr(z, 27)) * _MUL2
    return z ^ _lsr(z, 31)


def _mix_int(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, stream: int) -> int:
    """Key of one random stream; a stream is one tensor (or one slice family)."""
    return _mix_int(_mix_int(seed * 0x9E3779B97F4A7C15 + 0x1234567) ^ (stream * 0xD1B54A32D192ED03))


def random_bits(seed: int, stream: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """64 random bits (as int64) for counters start .. start+count-1 of a stream."""
    key = _as_i64(stream_key(seed, stream))
    ctr = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix((ctr + 1) * _GOLDEN + key)


def uniform_ints(seed: int, stream: int, count: int, lo: int, hi: int) -> np.ndarray:
    """count integers uniform in [lo, hi] (inclusive), host side."""
    bits = random_bits(seed, stream, 0, count)
    u = (_lsr(bits, 11).to(torch.float64) + 0.5) / float(1 << 53)
    return (lo + torch.floor(u * (hi - lo + 1)).to(torch.int64)).clamp_(lo, hi).numpy()


def uniform_unit(seed: int, stream: int, count: int) -> np.ndarray:
    bits = random_bits(seed, stream, 0, count)
    return ((_lsr(bits, 11).to(torch.float64) + 0.5) / float(1 << 53)).numpy()


def permutation(seed: int, stream: int, n: int) -> np.ndarray:
    """Seeded permutation of 0..n-1 (sort of random keys; ties broken by index)."""
    bits = random_bits(seed, stream, 0, n)
    return torch.argsort(_lsr(bits, 1), stable=True).numpy().astype(np.int64)


def normal_bf16(seed: int, stream: int, start: int, count: int, sigma: float, mean: float = 0.0,
                device="cpu") -> torch.Tensor:
    """count samples of N(mean, sigma^2), Box-Muller in fp64, rounded fp64->fp32->bf16 (RNE)."""
    bits = random_bits(seed, stream, start, count, device=device)
    u1 = (_lsr(bits, 32).to(torch.float64) + 0.5) / 4294967296.0
    u2 = ((bits & 0xFFFFFFFF).to(torch.float64) + 0.5) / 4294967296.0
    z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
    return (z * sigma + mean).to(torch.float32).to(torch.bfloat16)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """uint16 bit patterns of a bf16 tensor, as a host numpy array."""
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


# ----------------------------------------------------------------------------
# stage shape
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class StageShape:
    """Shape of one pipeline stage (a contiguous share of decoder layers)."""
    name: str
    num_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    intermediate: int
    page_size: int = PAGE
    rms_eps: float = 1e-6
    rope_theta: float = 10000.0
    has_qkv_bias: bool = False

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def n_qkv(self) -> int:
        return self.q_dim + 2 * self.kv_dim

    @property
    def weight_elems_per_layer(self) -> int:
        H, I = self.hidden, self.intermediate
        return H * self.n_qkv + self.q_dim * H + 3 * H * I

    @property
    def gemm_flop_per_token_layer(self) -> int:
        return 2 * self.weight_elems_per_layer

    @property
    def kv_bytes_per_token_layer(self) -> int:
        return 2 * self.kv_dim * 2


SHAPES: Dict[str, StageShape] = {
    "tiny": StageShape("tiny", 1, 256, 4, 2, 64, 688),
    "llama3_8b_pp4": StageShape("llama3_8b_pp4", 8, 4096, 32, 8, 128, 14336),
    "qwen25_14b_pp4": StageShape("qwen25_14b_pp4", 12, 5120, 40, 8, 128, 13824),
    "qwen25_32b_pp4": StageShape("qwen25_32b_pp4", 16, 5120, 64, 8, 128, 27648),
    "llama3_70b_pp4": StageShape("llama3_70b_pp4", 20, 8192, 64, 8, 128, 28672),
}

# stream ids ---------------------------------------------------------------
_ST_HIDDEN = 1
_ST_BATCH = 2
_ST_PERM = 3
_ST_POOL_K = 10
_ST_POOL_V = 11
_ST_LAYER0 = 1000  # + 32*layer + tensor kind
_W_KINDS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "norm1", "norm2", "bq", "bk", "bv")


def weight_shapes(shape: StageShape) -> Dict[str, Tuple[int, ...]]:
    """Row-major [out_features, in_features] matrices and the two norm gains of one layer."""
    H, I = shape.hidden, shape.intermediate
    s = {
        "wq": (shape.q_dim, H), "wk": (shape.kv_dim, H), "wv": (shape.kv_dim, H),
        "wo": (H, shape.q_dim), "wgate": (I, H), "wup": (I, H), "wdown": (H, I),
        "norm1": (H,), "norm2": (H,),
    }
    if shape.has_qkv_bias:
        s.update({"bq": (shape.q_dim,), "bk": (shape.kv_dim,), "bv": (shape.kv_dim,)})
    return s


def make_layer_weights(shape: StageShape, seed: int, layer: int, device="cpu") -> Dict[str, torch.Tensor]:
    """bf16 tensors of one layer: matrices N(0, 0.02^2), gains 1 + 0.1 N(0,1), biases N(0, 0.02^2)."""
    out = {}
    for name, shp in weight_shapes(shape).items():
        stream = _ST_LAYER0 + 32 * layer + _W_KINDS.index(name)
        n = int(np.prod(shp))
        if name.startswith("norm"):
            t = normal_bf16(seed, stream, 0, n, 0.1, 1.0, device=device)
        else:
            t = normal_bf16(seed, stream, 0, n, 0.02, 0.0, device=device)
        out[name] = t.reshape(shp)
    return out


def make_hidden(shape: StageShape, seed: int, num_tokens: int, device="cpu") -> torch.Tensor:
    """Stage input activations [T, H] bf16 ~ N(0,1)."""
    return normal_bf16(seed, _ST_HIDDEN, 0, num_tokens * shape.hidden, 1.0, device=device).reshape(
        num_tokens, shape.hidden)


# ----------------------------------------------------------------------------
# batches
# ----------------------------------------------------------------------------
@dataclass
class Batch:
    """One hybrid micro-batch: per sequence the new-token count and the cached length.

    Token rows are packed in sequence order.  block_tables[s, b] is the physical page of
    logical page b of sequence s (valid for ceil((cached+new)/page) entries, -1 after).
    """
    new_tokens: np.ndarray          # int32 [S]
    cached_len: np.ndarray          # int32 [S]
    block_tables: np.ndarray        # int32 [S, max_blocks_per_seq]
    num_blocks: int                 # physical pages in the pool
    label: str = ""

    @property
    def num_seqs(self) -> int:
        return int(self.new_tokens.shape[0])

    @property
    def num_tokens(self) -> int:
        return int(self.new_tokens.sum())

    @property
    def row_offsets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.new_tokens)]).astype(np.int64)

    def subset(self, seq_ids, new_tokens: Optional[List[int]] = None) -> "Batch":
        """The same sequences (optionally with fewer leading new tokens), same pages."""
        seq_ids = list(seq_ids)
        nt = self.new_tokens[seq_ids].copy()
        if new_tokens is not None:
            nt = np.asarray(new_tokens, dtype=np.int32)
        return Batch(nt.astype(np.int32), self.cached_len[seq_ids].copy(),
                     self.block_tables[seq_ids].copy(), self.num_blocks, self.label + ":subset")


def _pages(tokens: int) -> int:
    return (tokens + PAGE - 1) // PAGE


def build_batch(seqs: List[Tuple[int, int]], seed: int, spare_blocks: int = 0,
                max_blocks_per_seq: Optional[int] = None, label: str = "",
                perm_stream: int = _ST_PERM) -> Batch:
    """seqs = [(new_tokens, cached_len), ...]; pages are handed out through a seeded permutation."""
    need = [_pages(n + c) for n, c in seqs]
    total = sum(need)
    num_blocks = total + spare_blocks
    perm = permutation(seed, perm_stream, num_blocks)
    width = max_blocks_per_seq or max(need)
    bt = np.full((len(seqs), width), -1, dtype=np.int32)
    at = 0
    for s, nb in enumerate(need):
        bt[s, :nb] = perm[at:at + nb]
        at += nb
    return Batch(np.array([n for n, _ in seqs], dtype=np.int32),
                 np.array([c for _, c in seqs], dtype=np.int32), bt, num_blocks, label)


def make_batch(name: str, seed: int = 0, index: int = 0) -> Batch:
    """The batch of a named configuration (index selects the batch of the 70B-shaped series)."""
    if name == "tiny":
        seqs = [(32, 0), (16, 48), (1, 17), (1, 31), (1, 40), (1, 64)]
        return build_batch(seqs, seed, spare_blocks=14, label=name)  # 18 used pages in a 32-page pool
    if name == "llama3_8b_pp4":
        c0 = int(uniform_ints(seed, _ST_BATCH, 1, 0, 2047)[0])
        dec = uniform_ints(seed, _ST_BATCH + 100, 256, 512, 4096)
        seqs = [(1792, c0)] + [(1, int(c)) for c in dec]
        return build_batch(seqs, seed, spare_blocks=64, label=name)
    if name == "qwen25_14b_pp4":
        u = uniform_unit(seed, _ST_BATCH, 512)
        c = np.floor(np.exp(math.log(1024.0) + u * (math.log(8192.0) - math.log(1024.0)))).astype(np.int64)
        seqs = [(1, int(x)) for x in np.clip(c, 1024, 8192)]
        return build_batch(seqs, seed, spare_blocks=64, label=name)
    if name == "qwen25_32b_pp4":
        dec = uniform_ints(seed, _ST_BATCH + 100, 64, 256, 4096)
        seqs = [(1024, 0), (1024, 1024), (1024, 3072), (1024, 6144)] + [(1, int(c)) for c in dec]
        return build_batch(seqs, seed, spare_blocks=64, label=name)
    if name == "llama3_70b_pp4":
        return make_series(name, seed)[index]
    raise KeyError(name)


def make_decode_only_batch(rows: int, seed: int = 0, lo: int = 1500, hi: int = 3500) -> Batch:
    """A small decode-only micro-batch -- what the paper's Eq. 4 leaves of the running requests per micro-batch when few
    are decoding: `rows` sequences with one new token each over cached lengths uniform in [lo, hi]."""
    c = uniform_ints(seed, _ST_BATCH + 300, rows, lo, hi)
    return build_batch([(1, int(x)) for x in c], seed, spare_blocks=64, label=f"decode_only_{rows}")


def make_series(name: str = "llama3_70b_pp4", seed: int = 0, count: int = 16,
                pool_decodes: int = 512) -> List[Batch]:
    """16 consecutive batches over one shared pool.

    A pool of pool_decodes decode sequences (cached lengths uniform in [512, 8192]) and, per
    batch, ceil(P/2048) near-equal prefill chunks (P uniform in [0, 4096]) over cached prefixes
    uniform in [0, 4096).  Batch b decodes the first D_b (uniform in [32, 512]) sequences of a
    seeded order of the pool.  All batches share one page numbering.
    """
    dec_c = uniform_ints(seed, _ST_BATCH + 100, pool_decodes, 512, 8192)
    P = uniform_ints(seed, _ST_BATCH + 200, count, 0, 4096)
    D = uniform_ints(seed, _ST_BATCH + 201, count, 32, 512)
    pre_c = uniform_ints(seed, _ST_BATCH + 202, 2 * count, 0, 4095)
    order = permutation(seed, _ST_BATCH + 203, pool_decodes)
    # page budget: decode pool (+1 token each) and, per batch, its own chunk pages
    chunks: List[List[Tuple[int, int]]] = []
    for b in range(count):
        p = int(P[b])
        k = (p + 2047) // 2048
        cs = []
        for j in range(k):
            n = p // k + (1 if j < p % k else 0)
            cs.append((n, int(pre_c[2 * b + j])))
        chunks.append(cs)
    all_seqs = [(1, int(c)) for c in dec_c]
    for cs in chunks:
        all_seqs += cs
    whole = build_batch(all_seqs, seed, spare_blocks=64, label=name)
    out = []
    at = pool_decodes
    for b in range(count):
        ids = [int(x) for x in order[: int(D[b])]]
        pre_ids = list(range(at, at + len(chunks[b])))
        at += len(chunks[b])
        sel = pre_ids + ids
        out.append(Batch(whole.new_tokens[sel].copy(), whole.cached_len[sel].copy(),
                         whole.block_tables[sel].copy(), whole.num_blocks, f"{name}[{b}]"))
    return out


# ----------------------------------------------------------------------------
# paged KV pool
# ----------------------------------------------------------------------------
def pool_elems_per_layer(shape: StageShape, num_blocks: int) -> int:
    return num_blocks * shape.n_kv_heads * shape.page_size * shape.head_dim


def kv_sigma(shape: StageShape) -> float:
    """Std of a K or V element produced by an N(0,0.02^2) projection of a unit-variance row."""
    return 0.02 * math.sqrt(shape.hidden)


def make_pool(shape: StageShape, seed: int, num_blocks: int, device="cpu",
              chunk_elems: int = 1 << 26) -> Tuple[torch.Tensor, torch.Tensor]:
    """K and V pools, every page filled with seeded bf16 values N(0, (0.02 sqrt(H))^2).

    Returned as flat bf16 tensors of num_layers * num_blocks * n_kv * page * head_dim elements
    each; the element order inside a page is the library's business (the fill is i.i.d., so
    it is the same distribution under any layout).
    """
    n = shape.num_layers * pool_elems_per_layer(shape, num_blocks)
    sig = kv_sigma(shape)
    pools = []
    for stream in (_ST_POOL_K, _ST_POOL_V):
        buf = torch.empty(n, dtype=torch.bfloat16, device=device)
        for start in range(0, n, chunk_elems):
            cnt = min(chunk_elems, n - start)
            buf[start:start + cnt] = normal_bf16(seed, stream, start, cnt, sig, device=device)
        pools.append(buf)
    return pools[0], pools[1]


# ----------------------------------------------------------------------------
# sub-batches over a compact copy of the pages they use (for sampled checks of large batches)
# ----------------------------------------------------------------------------
def compact_subset(shape: StageShape, batch: Batch, seq_ids, new_tokens, k_pool: torch.Tensor,
                   v_pool: torch.Tensor):
    """Selects sequences (optionally only their first new tokens) and gathers the pages they own.

    Rows of a sequence depend only on that sequence's own rows and pages, and the first m rows of a
    chunk do not depend on its later rows, so the sub-batch reproduces those rows of the full batch.
    Returns (sub_batch with pages renumbered 0..n-1, k_bits, v_bits, page_ids): the pools are host
    uint16 arrays laid out [layer][page][...] like the originals; page_ids are the original ids.
    """
    sub = batch.subset(seq_ids, new_tokens)
    ids: List[int] = []
    bt = np.full_like(sub.block_tables, -1)
    for s in range(sub.num_seqs):
        nb = _pages(int(sub.new_tokens[s]) + int(sub.cached_len[s]))
        bt[s, :nb] = np.arange(len(ids), len(ids) + nb)
        ids += [int(x) for x in sub.block_tables[s, :nb]]
    per_page = shape.n_kv_heads * shape.page_size * shape.head_dim
    idx = torch.tensor(ids, dtype=torch.int64, device=k_pool.device)
    out = []
    for pool in (k_pool, v_pool):
        view = pool.view(shape.num_layers, batch.num_blocks, per_page)
        out.append(bf16_bits(view.index_select(1, idx)).reshape(-1).copy())
    return Batch(sub.new_tokens, sub.cached_len, bt, len(ids), sub.label), out[0], out[1], np.array(ids)
