"""Plumbing shared by the GPU parity tests: run the HIP stage through the C ABI on synthetic inputs."""
from __future__ import annotations

import numpy as np
import torch

from paper_2504_14775_amd import binding as B
from paper_2504_14775_amd import synth

DEV = "cuda"


def to_dev_bits(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns (host) -> bf16 tensor on the GPU, bits preserved."""
    return torch.from_numpy(bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)


def tiled_bits(bits: np.ndarray) -> np.ndarray:
    """A row-major [n][k] matrix in the weight layout the GEMM operations take (stated in include/gllm_stage.h): blocks
    of 64 rows x 64 columns, each contiguous and row-major inside, ordered [row block][column block].  Returned with
    the shape [n][k] the operations expect of the buffer."""
    n, k = bits.shape
    assert n % 64 == 0 and k % 64 == 0
    return np.ascontiguousarray(bits.reshape(n // 64, 64, k // 64, 64).transpose(0, 2, 1, 3)).reshape(n, k)


def to_dev_weight(bits: np.ndarray) -> torch.Tensor:
    return to_dev_bits(tiled_bits(bits))


def bits_of(t: torch.Tensor) -> np.ndarray:
    return synth.bf16_bits(t)


class GpuStage:
    """A stage with weights loaded; pools are bound per run."""

    def __init__(self, shape, weights_bits, batches, alias_check=True):
        self.shape = shape
        self.stage = B.stage_for_batches(shape, batches)
        self.stage.set_alias_check(alias_check)
        for l, w in enumerate(weights_bits):
            dev = {k: to_dev_bits(v) for k, v in w.items()}
            self.stage.load_layer(l, dev)
        torch.cuda.synchronize()

    def run(self, batch, k_pool: torch.Tensor, v_pool: torch.Tensor, hidden: torch.Tensor, want_f32=True):
        T = batch.num_tokens
        out = torch.empty(T, self.shape.hidden, dtype=torch.bfloat16, device=DEV)
        out32 = torch.empty(T, self.shape.hidden, dtype=torch.float32, device=DEV) if want_f32 else None
        self.stage.bind_kv_pool(k_pool, v_pool, batch.num_blocks)
        self.stage.forward(batch.new_tokens, batch.cached_len, batch.block_tables, hidden, out, out32)
        torch.cuda.synchronize()
        return out, out32


def parity_report(name, y_bf16_bits, y_f32, ref):
    """The literal and the scale-aware error figures of one comparison."""
    from oracle import bf16_to_f64, f64_to_bf16
    y16 = bf16_to_f64(y_bf16_bits)
    rms = float(np.sqrt((ref ** 2).mean()))
    rep = {
        "max_abs_bf16": float(np.abs(y16 - ref).max()),
        "mean_rel_bf16": float(np.abs(y16 - ref).sum() / np.abs(ref).sum()),
        "floor_max_abs": float(np.abs(bf16_to_f64(f64_to_bf16(ref)) - ref).max()),
        "rms_ref": rms, "max_ref": float(np.abs(ref).max()),
    }
    if y_f32 is not None:
        rep["max_abs_f32"] = float(np.abs(y_f32.astype(np.float64) - ref).max())
        rep["max_abs_f32_scaled"] = rep["max_abs_f32"] / max(1.0, rms)
    print(f"[parity] {name}: " + ", ".join(f"{k}={v:.4g}" for k, v in rep.items()), flush=True)
    return rep
