"""Shared test plumbing: synthetic inputs as host numpy arrays (bf16 as uint16 bits)."""
from __future__ import annotations

import dataclasses

import numpy as np

from paper_2504_14775_amd import synth


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
