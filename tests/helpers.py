"""Shared test plumbing: synthetic inputs as host numpy arrays (bf16 as uint16 bits)."""
from __future__ import annotations

import sys

import numpy as np

from paper_2504_14775_amd import synth


_capture_manager = None          # pytest's capture manager, set by conftest.pytest_configure


def say(msg: str) -> None:
    """A progress line of a long test: printed as usual (pytest shows it with a failure) and, while pytest captures
    output, also written to the real stderr, so that whoever watches the run sees that it is alive."""
    print(msg, flush=True)
    cm = _capture_manager
    if cm is not None and cm.is_globally_capturing():
        with cm.global_and_fixture_disabled():
            sys.stderr.write(msg + "\n")
            sys.stderr.flush()


def layer_weights_np(shape, seed, layers=None):
    out = []
    for l in range(shape.num_layers if layers is None else layers):
        w = synth.make_layer_weights(shape, seed, l)
        out.append({k: synth.bf16_bits(v) for k, v in w.items()})
    return out


def hidden_np(shape, seed, T):
    return synth.bf16_bits(synth.make_hidden(shape, seed, T))


def pool_np(shape, seed, num_blocks):
    k, v = synth.make_pool(shape, seed, num_blocks)
    return synth.bf16_bits(k).copy(), synth.bf16_bits(v).copy()


def small_shape(**kw):
    base = dict(name="unit", num_layers=1, hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16,
                intermediate=96)
    base.update(kw)
    return synth.StageShape(**base)


def error_metrics(y, ref):
    """max abs error, sum|d|/sum|ref|, rms(ref)."""
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    d = np.abs(y - ref)
    return float(d.max()), float(d.sum() / max(np.abs(ref).sum(), 1e-300)), float(np.sqrt((ref ** 2).mean()))


def written_mask(shape, batch):
    """Boolean mask over one flat K (or V) pool: True where this batch's new tokens must be stored.

    Written from the interface's statement of the layout, independently of oracle and library:
    position p of sequence s -> page block_tables[s][p // 16], slot p % 16, every layer, KV head and dim;
    K element (dim e) at (e // 8) * 128 + slot * 8 + e % 8, V element at e * 16 + slot inside the
    (page, head) block of head_dim * 16 elements.
    """
    ps, d, nkv = shape.page_size, shape.head_dim, shape.n_kv_heads
    per_layer = synth.pool_elems_per_layer(shape, batch.num_blocks)
    mk = np.zeros(shape.num_layers * per_layer, dtype=bool)
    mv = np.zeros_like(mk)
    e = np.arange(d)
    for s in range(batch.num_seqs):
        for i in range(int(batch.new_tokens[s])):
            p = int(batch.cached_len[s]) + i
            page, slot = int(batch.block_tables[s, p // ps]), p % ps
            for l in range(shape.num_layers):
                for h in range(nkv):
                    base = l * per_layer + (page * nkv + h) * ps * d
                    mk[base + (e // 8) * (ps * 8) + slot * 8 + e % 8] = True
                    mv[base + e * ps + slot] = True
    return mk, mv
