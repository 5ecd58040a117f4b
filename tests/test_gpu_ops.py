"""GPU parity of the single operations exported by the C ABI against the oracle's steps."""
import numpy as np
import pytest
import torch

import oracle
from paper_2504_14775_amd import binding as B
from paper_2504_14775_amd import synth
from gpu_util import DEV, bits_of, tiled_bits, to_dev_bits, to_dev_weight

pytestmark = pytest.mark.gpu


def rand_bits(seed, stream, shape, sigma):
    n = int(np.prod(shape))
    return synth.bf16_bits(synth.normal_bf16(seed, stream, 0, n, sigma)).reshape(shape)


def padded_rows(bits, rows):
    out = np.zeros((rows, bits.shape[1]), dtype=np.uint16)
    out[: bits.shape[0]] = bits
    return out


@pytest.mark.parametrize("tile", [-1, 0, 1, 2, 3, 6, 7, 10])
@pytest.mark.parametrize("M,N,K", [(1, 256, 64), (52, 512, 256), (300, 768, 192), (257, 1280, 704), (1024, 256, 2048)])
def test_gemm_store_and_add(M, N, K, tile):
    print(f"gemm store/add M={M} N={N} K={K} tile={tile}", flush=True)
    a = rand_bits(1, 1, (M, K), 1.0)
    w = rand_bits(1, 2, (N, K), 0.05)
    ref = oracle.linear(oracle.bf16_to_f64(a), w)
    Mp = (M + 255) // 256 * 256
    da, dw = to_dev_bits(padded_rows(a, Mp)), to_dev_weight(w)
    out = torch.full((M, N), 7.0, dtype=torch.float32, device=DEV)
    B.gllm_op_gemm_bf16(da, dw, out, M, N, K, B.GEMM_STORE_F32, tile)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    scale = np.abs(ref).max()
    assert np.abs(got - ref).max() <= 2e-5 * scale + 1e-6
    B.gllm_op_gemm_bf16(da, dw, out, M, N, K, B.GEMM_ADD_F32, tile)
    torch.cuda.synchronize()
    got2 = out.cpu().numpy().astype(np.float64)
    assert np.abs(got2 - 2 * ref).max() <= 4e-5 * scale + 1e-6


@pytest.mark.parametrize("tile", [-1, 0, 1, 2, 3, 6, 7, 10])
@pytest.mark.parametrize("M,I,K", [(52, 768, 256), (130, 128, 128), (300, 1408, 320)])
def test_gemm_swiglu(M, I, K, tile):
    print(f"gemm swiglu M={M} I={I} K={K} tile={tile}", flush=True)
    a = rand_bits(2, 1, (M, K), 1.0)
    wg = rand_bits(2, 2, (I, K), 0.08)
    wu = rand_bits(2, 3, (I, K), 0.08)
    x = oracle.bf16_to_f64(a)
    ref = oracle.swiglu(oracle.linear(x, wg), oracle.linear(x, wu))
    # interleave as the ABI states: groups of 64 rows = 32 gate rows then the 32 matching up rows
    assert I % 128 == 0
    packed = np.zeros((2 * I, K), dtype=np.uint16)
    for blk in range(I // 32):
        packed[64 * blk: 64 * blk + 32] = wg[32 * blk: 32 * blk + 32]
        packed[64 * blk + 32: 64 * blk + 64] = wu[32 * blk: 32 * blk + 32]
    Mp = (M + 255) // 256 * 256
    out = torch.zeros((M, I), dtype=torch.bfloat16, device=DEV)
    B.gllm_op_gemm_bf16(to_dev_bits(padded_rows(a, Mp)), to_dev_weight(packed), out, M, 2 * I, K, B.GEMM_SWIGLU_BF16, tile)
    torch.cuda.synchronize()
    got = oracle.bf16_to_f64(bits_of(out))
    err = np.abs(got - ref)
    assert np.all(err <= np.abs(ref) * 2.0 ** -7 + 1e-4), float(err.max())


@pytest.mark.parametrize("T,H", [(3, 256), (52, 4096), (17, 5120)])
def test_rmsnorm(T, H):
    print(f"rmsnorm T={T} H={H}", flush=True)
    x = synth.normal_bf16(3, 1, 0, T * H, 2.0).to(torch.float32).reshape(T, H) * 1.37
    gamma = rand_bits(3, 2, (H,), 0.5)
    ref = oracle.rmsnorm(x.numpy().astype(np.float64), gamma, 1e-6)
    h = torch.empty((T, H), dtype=torch.bfloat16, device=DEV)
    B.gllm_op_rmsnorm(x.to(DEV), to_dev_bits(gamma), h, 1e-6)
    torch.cuda.synchronize()
    got = oracle.bf16_to_f64(bits_of(h))
    assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -8 * 1.01 + 1e-6)


@pytest.mark.parametrize("M,N,K", [(300, 768, 192), (2, 192, 64), (513, 1536, 128)])
def test_gemm_256x192_tile(M, N, K):
    print(f"gemm 256x192 tile M={M} N={N} K={K}", flush=True)
    a = rand_bits(6, 1, (M, K), 1.0)
    w = rand_bits(6, 2, (N, K), 0.05)
    ref = oracle.linear(oracle.bf16_to_f64(a), w)
    Mp = (M + 255) // 256 * 256
    out = torch.full((M, N), 3.0, dtype=torch.float32, device=DEV)
    wpad = np.zeros(((N + 255) // 256 * 256, K), dtype=np.uint16); wpad[:N] = w
    B.gllm_op_gemm_bf16(to_dev_bits(padded_rows(a, Mp)), to_dev_weight(wpad), out, M, N, K, B.GEMM_STORE_F32, 5)
    B.gllm_op_gemm_bf16(to_dev_bits(padded_rows(a, Mp)), to_dev_weight(wpad), out, M, N, K, B.GEMM_ADD_F32, 5)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.abs(got - 2 * ref).max() <= 4e-5 * np.abs(ref).max() + 1e-6


@pytest.mark.parametrize("rowmix", [8, 12])
@pytest.mark.parametrize("M", [257, 300, 320, 384, 600, 832])
def test_gemm_row_mixed_launch(M, rowmix):
    """Whole bands of 256 rows as 256x256 tiles plus a last band of 64 (up to 64 rows left) or 128 rows: store, add,
    SwiGLU and split-K planes; tile 12 is the same with a third LDS stage for the weight tile."""
    N, K = 768, 384
    print(f"gemm row-mixed launch M={M} tile={rowmix}", flush=True)
    a = rand_bits(9, 1, (M, K), 1.0)
    w = rand_bits(9, 2, (N, K), 0.05)
    ref = oracle.linear(oracle.bf16_to_f64(a), w)
    Mp = (M + 255) // 256 * 256
    da, dw = to_dev_bits(padded_rows(a, Mp)), to_dev_weight(w)
    out = torch.full((M, N), 7.0, dtype=torch.float32, device=DEV)
    B.gllm_op_gemm_bf16(da, dw, out, M, N, K, B.GEMM_STORE_F32, rowmix)
    B.gllm_op_gemm_bf16(da, dw, out, M, N, K, B.GEMM_ADD_F32, rowmix)
    planes = torch.full((2, M, N), 9.0, dtype=torch.float32, device=DEV)
    B.gllm_op_gemm_bf16_splitk(da, dw, planes, M, N, K, rowmix, 2)
    torch.cuda.synchronize()
    scale = np.abs(ref).max()
    assert np.abs(out.cpu().numpy().astype(np.float64) - 2 * ref).max() <= 4e-5 * scale + 1e-6
    assert np.abs(planes.cpu().numpy().astype(np.float64).sum(axis=0) - ref).max() <= 2e-5 * scale + 1e-6
    # SwiGLU: the same matrix read as 384 gate/up pairs
    I = N // 2
    wg, wu = rand_bits(9, 3, (I, K), 0.08), rand_bits(9, 4, (I, K), 0.08)
    packed = np.zeros((2 * I, K), dtype=np.uint16)
    for blk in range(I // 32):
        packed[64 * blk: 64 * blk + 32] = wg[32 * blk: 32 * blk + 32]
        packed[64 * blk + 32: 64 * blk + 64] = wu[32 * blk: 32 * blk + 32]
    x = oracle.bf16_to_f64(a)
    ref_s = oracle.swiglu(oracle.linear(x, wg), oracle.linear(x, wu))
    act = torch.zeros((M, I), dtype=torch.bfloat16, device=DEV)
    B.gllm_op_gemm_bf16(da, to_dev_weight(packed), act, M, 2 * I, K, B.GEMM_SWIGLU_BF16, rowmix)
    torch.cuda.synchronize()
    err = np.abs(oracle.bf16_to_f64(bits_of(act)) - ref_s)
    assert np.all(err <= np.abs(ref_s) * 2.0 ** -7 + 1e-4), float(err.max())


@pytest.mark.parametrize("M", [257, 270, 288])
def test_gemm_288_row_tile(M):
    """All of 257..288 rows in one band of 288x192 tiles (six waves): store, add and split-K planes; refused outside
    that row range, for other column counts and for SwiGLU."""
    N, K = 576, 384
    print(f"gemm 288x192 tile M={M}", flush=True)
    a = rand_bits(10, 1, (M, K), 1.0)
    w = rand_bits(10, 2, (N, K), 0.05)
    ref = oracle.linear(oracle.bf16_to_f64(a), w)
    da, dw = to_dev_bits(padded_rows(a, 512)), to_dev_weight(w)
    out = torch.full((M, N), 7.0, dtype=torch.float32, device=DEV)
    B.gllm_op_gemm_bf16(da, dw, out, M, N, K, B.GEMM_STORE_F32, 9)
    B.gllm_op_gemm_bf16(da, dw, out, M, N, K, B.GEMM_ADD_F32, 9)
    planes = torch.full((2, M, N), 9.0, dtype=torch.float32, device=DEV)
    B.gllm_op_gemm_bf16_splitk(da, dw, planes, M, N, K, 9, 2)
    torch.cuda.synchronize()
    scale = np.abs(ref).max()
    assert np.abs(out.cpu().numpy().astype(np.float64) - 2 * ref).max() <= 4e-5 * scale + 1e-6
    assert np.abs(planes.cpu().numpy().astype(np.float64).sum(axis=0) - ref).max() <= 2e-5 * scale + 1e-6
    for m, n, mode in ((256, N, B.GEMM_STORE_F32), (289, N, B.GEMM_STORE_F32), (M, 512, B.GEMM_STORE_F32), (M, 768, B.GEMM_SWIGLU_BF16)):
        with pytest.raises(B.GllmError) as e:
            B.gllm_op_gemm_bf16(da, to_dev_weight(rand_bits(10, 3, (768, K), 0.05)), torch.empty(512, 768, device=DEV), m, n, K, mode, 9)
        assert e.value.status == -7          # GLLM_E_UNSUPPORTED


def test_gemm_row_mixed_launch_refuses_shapes_without_a_short_last_band():
    a = torch.zeros(1024, 128, dtype=torch.bfloat16, device=DEV)
    w = torch.zeros(256, 128, dtype=torch.bfloat16, device=DEV)
    for M in (100, 256, 512, 400, 700):                      # no whole band, nothing left over, more than 128 rows left over
        with pytest.raises(B.GllmError) as e:
            B.gllm_op_gemm_bf16(a, w, torch.empty(M, 256, device=DEV), M, 256, 128, B.GEMM_STORE_F32, 8)
        assert e.value.status == -7          # GLLM_E_UNSUPPORTED


@pytest.mark.parametrize("tile", [-1, 4, 11])
@pytest.mark.parametrize("mode", ["store", "swiglu"])
def test_gemm_mixed_tile_launch(mode, tile):
    """A grid whose last round of 256x256 tiles would be partial: 320 tiles -> 256 big + 128 half-width tiles."""
    M, N, K = 500, 40960, 128
    print(f"gemm mixed launch mode={mode} tile={tile}", flush=True)
    a = rand_bits(5, 1, (M, K), 1.0)
    x = oracle.bf16_to_f64(a)
    Mp = (M + 255) // 256 * 256
    if mode == "store":
        w = rand_bits(5, 2, (N, K), 0.05)
        ref = oracle.linear(x, w)
        out = torch.zeros((M, N), dtype=torch.float32, device=DEV)
        B.gllm_op_gemm_bf16(to_dev_bits(padded_rows(a, Mp)), to_dev_weight(w), out, M, N, K, B.GEMM_STORE_F32, tile)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        assert np.abs(got - ref).max() <= 2e-5 * np.abs(ref).max() + 1e-6
    else:
        I = N // 2
        wg = rand_bits(5, 3, (I, K), 0.08)
        wu = rand_bits(5, 4, (I, K), 0.08)
        ref = oracle.swiglu(oracle.linear(x, wg), oracle.linear(x, wu))
        packed = np.zeros((N, K), dtype=np.uint16)
        pk = packed.reshape(I // 32, 2, 32, K)
        pk[:, 0] = wg.reshape(I // 32, 32, K)
        pk[:, 1] = wu.reshape(I // 32, 32, K)
        out = torch.zeros((M, I), dtype=torch.bfloat16, device=DEV)
        B.gllm_op_gemm_bf16(to_dev_bits(padded_rows(a, Mp)), to_dev_weight(packed), out, M, N, K, B.GEMM_SWIGLU_BF16, tile)
        torch.cuda.synchronize()
        got = oracle.bf16_to_f64(bits_of(out))
        assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -7 + 1e-4)


@pytest.mark.parametrize("tile,splits", [(0, 2), (3, 2), (3, 4), (2, 4), (-1, 2), (6, 2), (7, 4), (10, 2), (10, 8)])
def test_gemm_split_k_planes_sum_to_the_product(tile, splits):
    M, N, K = 300, 512, 1024
    print(f"gemm split-K tile={tile} splits={splits}", flush=True)
    a = rand_bits(7, 1, (M, K), 1.0)
    w = rand_bits(7, 2, (N, K), 0.05)
    ref = oracle.linear(oracle.bf16_to_f64(a), w)
    Mp = (M + 255) // 256 * 256
    planes = torch.full((splits, M, N), 9.0, dtype=torch.float32, device=DEV)
    B.gllm_op_gemm_bf16_splitk(to_dev_bits(padded_rows(a, Mp)), to_dev_weight(w), planes, M, N, K, tile, splits)
    torch.cuda.synchronize()
    got = planes.cpu().numpy().astype(np.float64)
    assert np.abs(got.sum(axis=0) - ref).max() <= 2e-5 * np.abs(ref).max() + 1e-6
    # each plane is the product over its own share of k
    x = oracle.bf16_to_f64(a)
    ks = K // splits
    part0 = oracle.linear(x[:, :ks], np.ascontiguousarray(w[:, :ks]))
    assert np.abs(got[0] - part0).max() <= 2e-5 * np.abs(part0).max() + 1e-6


def test_gemm_third_weight_stage_changes_no_bit():
    """Tiles 10 / 11 / 12 are tiles 3 / 4 / 8 with one more LDS stage for the weight tile: the same products in the same
    order, so the results must be bit-identical -- also with few k-steps (fewer than stages) and with split-K."""
    for M, N, K, pair, splits in ((700, 1024, 64, (3, 10), 1), (700, 1024, 128, (3, 10), 1), (520, 768, 1152, (3, 10), 3),
                                  (300, 768, 640, (8, 12), 2), (500, 40960, 192, (4, 11), 1)):
        a = to_dev_bits(padded_rows(rand_bits(11, 1, (M, K), 1.0), (M + 255) // 256 * 256))
        w = to_dev_weight(rand_bits(11, 2, (N, K), 0.05))
        outs = []
        for tile in pair:
            planes = torch.full((splits, M, N), 5.0, dtype=torch.float32, device=DEV)
            B.gllm_op_gemm_bf16_splitk(a, w, planes, M, N, K, tile, splits)
            outs.append(planes)
        torch.cuda.synchronize()
        assert torch.equal(outs[0], outs[1]), (M, N, K, pair, splits)


def test_pack_weight_writes_the_documented_tiled_layout():
    """gllm_op_pack_weight against the layout as the header states it (gpu_util.tiled_bits), bit for bit: a whole matrix,
    and a part of a wider one (row stride above k); then the product on a leading part of the packed k range."""
    w = rand_bits(12, 1, (320, 448), 0.05)
    out = torch.zeros(320 * 448, dtype=torch.bfloat16, device=DEV)
    B.gllm_op_pack_weight(to_dev_bits(w), out)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(out).reshape(320, 448), tiled_bits(w))
    part = torch.zeros(128 * 192, dtype=torch.bfloat16, device=DEV)
    B.gllm_op_pack_weight(to_dev_bits(w)[64:192, :192], part)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(part).reshape(128, 192), tiled_bits(np.ascontiguousarray(w[64:192, :192])))
    for bad in (to_dev_bits(w)[:100], to_dev_bits(w)[:, :100]):          # rows / columns that are no multiple of 64
        with pytest.raises(B.GllmError) as e:
            B.gllm_op_pack_weight(bad, out)
        assert e.value.status == -7          # GLLM_E_UNSUPPORTED
    M, N, K, k = 70, 256, 448, 192
    a = rand_bits(12, 2, (M, K), 1.0)
    wn = rand_bits(12, 3, (N, K), 0.05)
    res = torch.zeros(M, N, dtype=torch.float32, device=DEV)
    B.gllm_op_gemm_bf16(to_dev_bits(padded_rows(a, 256)), to_dev_weight(wn), res, M, N, k, B.GEMM_STORE_F32, -1)
    torch.cuda.synchronize()
    ref = oracle.linear(oracle.bf16_to_f64(a)[:, :k], np.ascontiguousarray(wn[:, :k]))
    assert np.abs(res.cpu().numpy() - ref).max() <= 2e-5 * np.abs(ref).max() + 1e-6
    with pytest.raises(B.GllmError):          # a k extent that is no multiple of 64
        B.gllm_op_gemm_bf16(to_dev_bits(padded_rows(a, 256)), to_dev_weight(wn), res, M, N, k, B.GEMM_STORE_F32, -1, ldw=200)
