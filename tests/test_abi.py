"""The C-ABI library loads and exports every function include/gllm_stage.h declares (no GPU needed)."""
import os
import re

import pytest

from paper_2504_14775_amd import binding as B
from paper_2504_14775_amd import synth

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "gllm_stage.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gllm_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    for n in ("gllm_stage_create", "gllm_stage_forward", "gllm_stage_load_layer", "gllm_stage_bind_kv_pool",
              "gllm_stage_bind_workspace", "gllm_stage_destroy", "gllm_last_error"):
        assert n in names


def test_library_exports_every_declared_function():
    lib = B.load_library()
    for n in declared_functions():
        assert hasattr(lib, n), n
    assert set(B.EXPORTS) == set(declared_functions())


def test_status_names_and_profile_classes():
    lib = B.load_library()
    for code, name in B.STATUS.items():
        assert lib.gllm_status_name(code).decode() == name
    n = lib.gllm_profile_num_classes()
    names = [lib.gllm_profile_class_name(i).decode() for i in range(n)]
    assert "gemm_gate_up_swiglu" in names and "attn_decode" in names and len(set(names)) == n


def test_create_rejects_bad_configs_before_touching_a_device():
    shape = synth.SHAPES["tiny"]
    import dataclasses
    for bad, status in [
        (dict(page_size=8), -7),
        (dict(head_dim=96), -7),
        (dict(n_q_heads=5), -7),
        (dict(hidden=200), -7),
        (dict(hidden=192), -7),          # a multiple of 64 but not of 128: the header states 128
        (dict(num_layers=0), -1),
    ]:
        cfg = B.make_config(dataclasses.replace(shape, **bad), 64, 8, 8, 128)
        with pytest.raises(B.GllmError) as e:
            B.Stage(cfg)
        assert e.value.status == status, (bad, e.value)
    cfg = B.make_config(shape, 64, 8, 4, 128)          # 4 pages cannot hold 128 positions
    with pytest.raises(B.GllmError) as e:
        B.Stage(cfg)
    assert e.value.status == -1


def test_gemm_planner_choices_are_launchable():
    """Host logic of the tile / split-K planner: whatever it picks must satisfy the launch rules of that tile
    (column multiple, split divides the 64-wide k-steps, splits only in store mode), for the stage shapes and a
    sweep of ragged row counts."""
    col_multiple = {0: 128, 1: 128, 2: 256, 3: 256, 4: 256, 5: 192, 6: 128, 7: 128, 8: 256, 9: 192, 10: 256, 11: 256, 12: 256}
    seen = set()
    for shape in synth.SHAPES.values():
        H, I = shape.hidden, shape.intermediate
        pad = lambda v, q: (v + q - 1) // q * q
        n_qkv = pad((shape.n_q_heads + 2 * shape.n_kv_heads) * shape.head_dim, 256)
        problems = [(n_qkv, pad(H, 64), 0), (pad(H, 256), pad(shape.n_q_heads * shape.head_dim, 64), 0),
                    (2 * pad(I, 256), pad(H, 64), 2), (pad(H, 256), pad(I, 256), 0)]
        for m in (1, 17, 128, 256, 257, 288, 289, 512, 1000, 2048, 2560, 4160):
            for n, k, mode in problems:
                tile, splits = B.gllm_op_gemm_plan(m, n, k, mode, 8)
                seen.add(tile)
                assert tile in col_multiple and n % col_multiple[tile] == 0, (shape.name, m, n, k, mode, tile)
                assert 1 <= splits <= 8 and (k // 64) % splits == 0
                if mode != 0:
                    assert splits == 1 and tile != 5
                if tile == 7:
                    assert m <= 64
                if tile in (8, 12):
                    assert m > 256 and 0 < m % 256 <= 128
                if tile == 9:
                    assert 256 < m <= 288 and mode == 0
                if tile in (10, 11, 12):      # the third weight stage: long k or few rows
                    assert (k // 64) // splits >= 80 or m <= 1024
                if tile in (4, 11):
                    tiles = ((m + 255) // 256) * (n // 256)
                    assert splits == 1 and tiles >= 256 and 0 < tiles % 256 <= 128
                assert B.gllm_op_gemm_plan(m, n, k, mode, 8) == (tile, splits)          # deterministic
                assert B.gllm_op_gemm_plan(m, n, k, mode, 1)[1] == 1                    # the cap is respected
    # big problems get 256x256 tiles (with a short last band where rows are left over; with a third weight stage for
    # long k or few rows), few rows the deep 128x128 or the 64x128 one
    assert {3, 6, 7, 8, 10, 12}.issubset(seen), seen
    # the vocabulary projection of a micro-batch of 256 decode rows plus one chunk end: one 288-row band
    assert B.gllm_op_gemm_plan(257, 128256, 4096, 0, 1) == (9, 1)
    assert B.gllm_op_gemm_plan(256, 128256, 4096, 0, 1)[0] == 10 and B.gllm_op_gemm_plan(289, 128256, 4096, 0, 1)[0] == 12
    assert B.gllm_op_gemm_plan(2048, 4096, 14336, 0, 8) == (10, 2) and B.gllm_op_gemm_plan(2048, 4096, 4096, 0, 8) == (3, 2)
    with pytest.raises(B.GllmError):
        B.gllm_op_gemm_plan(128, 100, 4096, 0, 8)
