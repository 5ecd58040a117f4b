"""gllm_head_logits_static (the projection to logits with its scratch in a fixed array inside the library, for callers
that cannot allocate) against gllm_head_logits (scratch in a bound workspace): the same kernels on the same inputs, so
the logits must agree bit for bit -- on two calls in a row, the second with fewer rows, then a third that needs the
288-row tile -- and sizes beyond the array are refused before anything is enqueued."""
import numpy as np
import pytest
import torch

from paper_2504_14775_amd import binding as B
from paper_2504_14775_amd import head as HD
from paper_2504_14775_amd import synth
from gpu_util import DEV, to_dev_bits

pytestmark = pytest.mark.gpu


def test_static_scratch_projection_equals_the_workspace_one_on_consecutive_calls():
    H, V, T = 4096, 32256, 700          # 32256 = 42 * 768: the 288 x 192 tile applies at 270 rows
    print(f"no-alloc logits H={H} V={V}", flush=True)
    gain = synth.bf16_bits(synth.normal_bf16(7, 1, 0, H, 0.1, 1.0))
    w = synth.normal_bf16(7, 2, 0, V * H, 0.02, 0.0, device=DEV).view(V, H)
    x = (torch.randn(T, H, generator=torch.Generator().manual_seed(8)) * 3.0).to(torch.float32).to(DEV)
    rng = np.random.default_rng(9)
    ref_head = HD.Head(H, V, 1024, 1e-6)                          # workspace bound
    head = HD.Head(H, V, 4, 1e-6, bind_workspace=False)           # no workspace at all; max_rows is not consulted
    ref_head.load(to_dev_bits(gain), w)
    head.load(to_dev_bits(gain), w)
    assert int(head.lib.gllm_head_static_scratch_bytes()) == 8 << 20
    for M in (600, 37, 270):                                      # a big call, a smaller one after it, the 288-row tile
        rows = torch.from_numpy(rng.integers(0, T, size=M).astype(np.int32)).to(DEV)
        want = torch.full((M, ref_head.padded_vocab), float("nan"), dtype=torch.float32, device=DEV)
        got = torch.full((M, head.padded_vocab), float("nan"), dtype=torch.float32, device=DEV)
        ref_head.logits(x, rows, want)
        head.logits_static(x, rows, got)
        torch.cuda.synchronize()
        assert not torch.isnan(want).any()
        assert torch.equal(got.view(torch.int32), want.view(torch.int32)), M
        print(f"  {M} rows: bit-identical", flush=True)
    # beyond the array: 1025 rows round up to 1280 x 4096 x 2 bytes = 10 MiB > 8 MiB
    rows = torch.zeros(1025, dtype=torch.int32, device=DEV)
    out = torch.zeros(1025, head.padded_vocab, dtype=torch.float32, device=DEV)
    with pytest.raises(B.GllmError) as e:
        head.logits_static(x, rows, out)
    assert e.value.status == -2 and "static scratch" in e.value.message
    torch.cuda.synchronize()
    assert not out.any()                                          # nothing was enqueued
    fresh = HD.Head(H, V, 4, 1e-6, bind_workspace=False)
    with pytest.raises(B.GllmError) as e:                         # weights not loaded
        fresh.logits_static(x, rows[:4], out[:4])
    assert e.value.status == -5
    for h in (ref_head, head, fresh):
        h.destroy()
