"""Pins for the oracle's individual steps: closed forms, special cases and brute force.

Each test is chosen so that a plausible slip in the oracle (a dropped term, a wrong sign or
index, a transposed operand) fails it.  None of them touches the HIP library.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2504_14775_amd import synth
from helpers import small_shape


def bits_of(x):
    """bf16 bits of float values through torch's own float32 -> bf16 RNE."""
    return synth.bf16_bits(torch.tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16))


# ------------------------------------------------------------------ bf16 rounding
def test_bf16_roundtrip_all_finite_patterns():
    bits = np.arange(0, 1 << 16, dtype=np.uint32).astype(np.uint16)
    vals = oracle.bf16_to_f64(bits)
    finite = np.isfinite(vals)
    back = oracle.f64_to_bf16(vals[finite])
    assert np.array_equal(back, bits[finite])


def test_bf16_rne_matches_torch_on_float32_inputs():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-20, 20, 200000))).astype(np.float32)
    assert np.array_equal(oracle.f64_to_bf16(x.astype(np.float64)), bits_of(x))


def test_bf16_ties_and_single_rounding_from_double():
    one = 1.0
    ulp = 2.0 ** -7           # bf16 spacing in [1,2)
    # exact ties go to the even significand
    assert oracle.f64_to_bf16(np.array([one + ulp / 2]))[0] == 0x3F80
    assert oracle.f64_to_bf16(np.array([one + 3 * ulp / 2]))[0] == 0x3F82
    # a double just above a tie must round up even though float32 rounding lands on the tie
    x = one + ulp / 2 + 2.0 ** -40
    assert np.float32(x) == np.float32(one + ulp / 2)
    assert oracle.f64_to_bf16(np.array([x]))[0] == 0x3F81
    # and just below the tie rounds down
    assert oracle.f64_to_bf16(np.array([one + ulp / 2 - 2.0 ** -40]))[0] == 0x3F80
    assert oracle.f64_to_bf16(np.array([-x]))[0] == 0xBF81


# ------------------------------------------------------------------ RMSNorm
def test_rmsnorm_constant_row_closed_form():
    H, eps = 48, 1e-6
    gamma = bits_of(np.linspace(0.5, 1.5, H))
    g = oracle.bf16_to_f64(gamma)
    for c in (0.25, -3.0, 1e-3):
        out = oracle.rmsnorm(np.full((2, H), c), gamma, eps)
        want = g * c / math.sqrt(c * c + eps)
        np.testing.assert_allclose(out[0], want, rtol=1e-14)
        np.testing.assert_allclose(out[1], want, rtol=1e-14)


def test_rmsnorm_no_mean_subtraction_and_unit_power():
    rng = np.random.default_rng(1)
    H = 64
    x = rng.standard_normal((5, H)) + 3.0          # a large mean must survive
    gamma = bits_of(np.ones(H))
    out = oracle.rmsnorm(x, gamma, 0.0)
    np.testing.assert_allclose((out ** 2).mean(axis=1), 1.0, rtol=1e-13)
    assert np.all(np.sign(out) == np.sign(x))
    # scale invariance for eps = 0 and row independence
    np.testing.assert_allclose(oracle.rmsnorm(7.5 * x, gamma, 0.0), out, rtol=1e-13)
    np.testing.assert_array_equal(oracle.rmsnorm(x[2:3], gamma, 0.0)[0], out[2])


def test_rmsnorm_eps_is_inside_the_root():
    H = 16
    x = np.zeros((1, H)); x[0, 0] = 4.0          # mean square = 1
    out = oracle.rmsnorm(x, bits_of(np.ones(H)), 3.0)
    assert out[0, 0] == pytest.approx(4.0 / math.sqrt(1.0 + 3.0), rel=1e-15)


# ------------------------------------------------------------------ linear
def test_linear_matches_library_matmul_non_square():
    rng = np.random.default_rng(2)
    T, K, N = 7, 130, 70                      # N spans no full column chunk; K not a multiple of 8
    x = rng.standard_normal((T, K))
    w = bits_of(rng.standard_normal((N, K)) * 0.1)
    b = bits_of(rng.standard_normal(N))
    want = x @ oracle.bf16_to_f64(w).T + oracle.bf16_to_f64(b)
    np.testing.assert_allclose(oracle.linear(x, w, b), want, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.linear(x, w), want - oracle.bf16_to_f64(b), rtol=1e-12, atol=1e-12)


def test_linear_wide_output_spans_several_column_chunks():
    rng = np.random.default_rng(3)
    T, K, N = 3, 40, 1100
    x = rng.standard_normal((T, K))
    w = bits_of(rng.standard_normal((N, K)))
    np.testing.assert_allclose(oracle.linear(x, w), x @ oracle.bf16_to_f64(w).T, rtol=1e-12, atol=1e-12)


def test_linear_selector_matrix_picks_columns():
    # W[n][k] = 1 iff k == perm[n]  =>  y[t][n] = x[t][perm[n]] exactly (orientation check)
    rng = np.random.default_rng(4)
    K, N = 12, 9
    perm = rng.permutation(K)[:N]
    w = np.zeros((N, K)); w[np.arange(N), perm] = 1.0
    x = rng.standard_normal((4, K))
    np.testing.assert_array_equal(oracle.linear(x, bits_of(w)), x[:, perm])


def test_linear_rows_do_not_depend_on_batch():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((9, 33))
    w = bits_of(rng.standard_normal((21, 33)))
    full = oracle.linear(x, w)
    np.testing.assert_array_equal(oracle.linear(x[4:5], w)[0], full[4])


# ------------------------------------------------------------------ RoPE
def test_rope_position_zero_is_identity():
    rng = np.random.default_rng(6)
    v = rng.standard_normal((3, 2, 8))
    np.testing.assert_array_equal(oracle.rope(v, [0, 0, 0], 10000.0), v)


def test_rope_unit_vectors_closed_form():
    d, base, p = 4, 100.0, 3
    # theta_0 = 1, theta_1 = base^(-2/4) = 0.1 ; pairs are (0,2) and (1,3)
    e = np.zeros((4, 1, d))
    for i in range(4):
        e[i, 0, i] = 1.0
    out = oracle.rope(e, [p] * 4, base)[:, 0, :]
    c0, s0, c1, s1 = math.cos(3.0), math.sin(3.0), math.cos(0.3), math.sin(0.3)
    want = np.array([[c0, 0, s0, 0],      # e0 -> first half keeps cos, partner gets +sin
                     [0, c1, 0, s1],
                     [-s0, 0, c0, 0],     # e2 -> contributes -sin to its partner in the first half
                     [0, -s1, 0, c1]])
    np.testing.assert_allclose(out, want, atol=1e-15)


def test_rope_preserves_pair_norms_and_relative_position():
    rng = np.random.default_rng(7)
    d = 16
    q = rng.standard_normal((1, 1, d)); k = rng.standard_normal((1, 1, d))
    r = oracle.rope(q, [1234], 10000.0)
    np.testing.assert_allclose(r[0, 0, :8] ** 2 + r[0, 0, 8:] ** 2, q[0, 0, :8] ** 2 + q[0, 0, 8:] ** 2,
                               rtol=1e-12)
    def score(pq, pk):
        return float((oracle.rope(q, [pq], 10000.0) * oracle.rope(k, [pk], 10000.0)).sum())
    assert score(40, 33) == pytest.approx(score(1007, 1000), rel=1e-9)
    assert score(7, 0) == pytest.approx(score(40, 33), rel=1e-9)
    assert abs(score(40, 33) - score(40, 30)) > 1e-3


def test_rope_each_row_uses_its_own_position_and_all_heads_rotate():
    rng = np.random.default_rng(8)
    v = rng.standard_normal((3, 3, 8))
    pos = [5, 0, 9]
    out = oracle.rope(v, pos, 10000.0)
    for t in range(3):
        for h in range(3):
            np.testing.assert_array_equal(out[t, h], oracle.rope(v[t:t + 1, h:h + 1], [pos[t]], 10000.0)[0, 0])
    np.testing.assert_array_equal(out[1], v[1])


# ------------------------------------------------------------------ SwiGLU
def test_swiglu_values():
    g = np.array([0.0, 1.0, -1.0, 30.0, -30.0])
    u = np.array([5.0, 2.0, 2.0, 1.0, 1.0])
    out = oracle.swiglu(g, u)
    assert out[0] == 0.0
    assert out[1] == pytest.approx(2.0 / (1.0 + math.exp(-1.0)), rel=1e-15)
    assert out[2] == pytest.approx(-2.0 / (1.0 + math.exp(1.0)), rel=1e-15)
    assert out[3] == pytest.approx(30.0, rel=1e-12)
    assert abs(out[4]) < 1e-11
    # silu(z) - silu(-z) = z
    z = np.linspace(-6, 6, 25)
    np.testing.assert_allclose(oracle.swiglu(z, np.ones_like(z)) - oracle.swiglu(-z, np.ones_like(z)), z, atol=1e-14)


# ------------------------------------------------------------------ token map / slots
def test_token_map_packs_rows_in_sequence_order():
    seq_of, pos_of = oracle.token_map([3, 1, 2], [0, 17, 5])
    assert seq_of.tolist() == [0, 0, 0, 1, 2, 2]
    assert pos_of.tolist() == [0, 1, 2, 17, 5, 6]


def _pool_layout_index(shape, num_pages, which, layer, page, h, slot, dim):
    """The pool layout as the interface states it, written out independently of the oracle."""
    ps, d = shape.page_size, shape.head_dim
    base = ((layer * num_pages + page) * shape.n_kv_heads + h) * ps * d
    if which == "k":
        return base + (dim // 8) * ps * 8 + slot * 8 + dim % 8
    return base + dim * ps + slot


def test_kv_write_slot_placement_tiny_config_edges():
    """Slot of position p is page_table[p // 16] * 16 + p % 16; nothing else may change."""
    shape = synth.SHAPES["tiny"]
    batch = synth.make_batch("tiny", seed=0)
    seq_of, pos_of = oracle.token_map(batch.new_tokens, batch.cached_len)
    T = len(seq_of)
    n = shape.num_layers * synth.pool_elems_per_layer(shape, batch.num_blocks)
    SENT = 0x7FC1
    kp = np.full(n, SENT, dtype=np.uint16); vp = np.full(n, SENT, dtype=np.uint16)
    # value encodes (row, head, dim) exactly in bf16: small integers
    k = np.zeros((T, shape.n_kv_heads, shape.head_dim)); v = np.zeros_like(k)
    for t in range(T):
        for h in range(shape.n_kv_heads):
            k[t, h, :] = (t % 64) + 1
            v[t, h, :] = -((t % 64) + 1)
    k[:, 1, :] += 64; v[:, 1, :] -= 64
    k[:, :, 5] = 200.0; v[:, :, 5] = -200.0         # marks dim 5
    oracle.kv_write(shape, 0, seq_of, pos_of, batch.block_tables, batch.num_blocks, k, v, kp, vp)
    expect_k = np.full(n, SENT, dtype=np.uint16); expect_v = expect_k.copy()
    kb, vb = bits_of(k), bits_of(v)
    for t in range(T):
        s, p = seq_of[t], pos_of[t]
        page = batch.block_tables[s, p // 16]
        for h in range(shape.n_kv_heads):
            for dim in range(shape.head_dim):
                expect_k[_pool_layout_index(shape, batch.num_blocks, "k", 0, page, h, p % 16, dim)] = kb[t, h, dim]
                expect_v[_pool_layout_index(shape, batch.num_blocks, "v", 0, page, h, p % 16, dim)] = vb[t, h, dim]
    assert np.array_equal(kp, expect_k)
    assert np.array_equal(vp, expect_v)
    # edges named by the configuration: c=64 -> slot 0 of a fresh 5th page, c=31 -> last slot of page 1,
    # c=17 -> slot 1 of page 1, the 16-over-48 chunk fills exactly logical page 3
    pos_by_seq = {s: [p for ss, p in zip(seq_of, pos_of) if ss == s] for s in range(6)}
    assert pos_by_seq[5] == [64] and 64 // 16 == 4 and 64 % 16 == 0
    assert pos_by_seq[3] == [31] and 31 % 16 == 15
    assert pos_by_seq[1] == list(range(48, 64))
    written = int((kp != SENT).sum())
    assert written == T * shape.n_kv_heads * shape.head_dim


def test_pool_index_functions_match_stated_layout():
    shape = small_shape(head_dim=16, n_kv_heads=3)
    for which in "kv":
        seen = set()
        for layer in range(2):
            for page in (0, 4):
                for h in range(3):
                    for slot in range(16):
                        for dim in range(16):
                            i = oracle.pool_index(shape, which, 5, layer, page, h, slot, dim)
                            assert i == _pool_layout_index(shape, 5, which, layer, page, h, slot, dim)
                            seen.add(i)
        assert len(seen) == 2 * 2 * 3 * 16 * 16


# ------------------------------------------------------------------ attention
def _fill_pool_from_dense(shape, num_pages, bt_row, K, V):
    """K, V: [n_pos, n_kv, d] bf16 bits -> pools holding them at the logical positions."""
    n = synth.pool_elems_per_layer(shape, num_pages)
    kp = np.zeros(n, dtype=np.uint16); vp = np.zeros(n, dtype=np.uint16)
    for p in range(K.shape[0]):
        for h in range(shape.n_kv_heads):
            for dim in range(shape.head_dim):
                kp[_pool_layout_index(shape, num_pages, "k", 0, bt_row[p // 16], h, p % 16, dim)] = K[p, h, dim]
                vp[_pool_layout_index(shape, num_pages, "v", 0, bt_row[p // 16], h, p % 16, dim)] = V[p, h, dim]
    return kp, vp


def _brute_force_attention(q, K, V, n_q, n_kv, first_pos):
    """Dense masked softmax in float64: q [n, n_q, d]; K, V [n_pos, n_kv, d] (float64)."""
    n, _, d = q.shape
    g = n_q // n_kv
    out = np.zeros_like(q)
    for h in range(n_q):
        S = q[:, h, :] @ K[:, h // g, :].T / math.sqrt(d)           # [n, n_pos]
        mask = np.arange(K.shape[0])[None, :] <= (first_pos + np.arange(n))[:, None]
        S = np.where(mask, S, -np.inf)
        P = np.exp(S - S.max(axis=1, keepdims=True))
        P /= P.sum(axis=1, keepdims=True)
        out[:, h, :] = P @ V[:, h // g, :]
    return out


@pytest.mark.parametrize("n_new,cached", [(37, 0), (5, 43), (1, 52), (16, 16)])
def test_attention_against_brute_force(n_new, cached):
    shape = small_shape(n_q_heads=6, n_kv_heads=2, head_dim=8)
    rng = np.random.default_rng(11)
    total = n_new + cached
    pages = (total + 15) // 16
    num_pages = pages + 3
    bt = rng.permutation(num_pages)[:pages].astype(np.int32)[None, :]
    Kb = bits_of(rng.standard_normal((total, 2, 8))); Vb = bits_of(rng.standard_normal((total, 2, 8)))
    kp, vp = _fill_pool_from_dense(shape, num_pages, bt[0], Kb, Vb)
    q = rng.standard_normal((n_new, 6, 8)) * 2.0
    seq_of = np.zeros(n_new, dtype=np.int32)
    pos_of = (cached + np.arange(n_new)).astype(np.int32)
    got = oracle.attention(shape, 0, seq_of, pos_of, bt, num_pages, q, kp, vp)
    want = _brute_force_attention(q, oracle.bf16_to_f64(Kb), oracle.bf16_to_f64(Vb), 6, 2, cached)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_attention_single_key_returns_that_value_exactly():
    shape = small_shape(n_q_heads=2, n_kv_heads=2, head_dim=8)
    rng = np.random.default_rng(12)
    Kb = bits_of(rng.standard_normal((1, 2, 8))); Vb = bits_of(rng.standard_normal((1, 2, 8)))
    bt = np.array([[2]], dtype=np.int32)
    kp, vp = _fill_pool_from_dense(shape, 4, bt[0], Kb, Vb)
    q = rng.standard_normal((1, 2, 8))
    got = oracle.attention(shape, 0, [0], [0], bt, 4, q, kp, vp)
    np.testing.assert_array_equal(got[0], oracle.bf16_to_f64(Vb)[0])


def test_attention_equal_keys_average_values_and_shift_invariance():
    shape = small_shape(n_q_heads=2, n_kv_heads=1, head_dim=8)
    rng = np.random.default_rng(13)
    n = 20
    key = bits_of(rng.standard_normal((1, 1, 8)))
    Kb = np.repeat(key, n, axis=0); Vb = bits_of(rng.standard_normal((n, 1, 8)))
    bt = np.array([[1, 0]], dtype=np.int32)
    kp, vp = _fill_pool_from_dense(shape, 2, bt[0], Kb, Vb)
    q = rng.standard_normal((1, 2, 8))
    got = oracle.attention(shape, 0, [0], [n - 1], bt, 2, q, kp, vp)
    want = oracle.bf16_to_f64(Vb)[:, 0, :].mean(axis=0)
    np.testing.assert_allclose(got[0, 0], want, rtol=1e-13)
    np.testing.assert_allclose(got[0, 1], want, rtol=1e-13)
    # scaling q rescales all (equal) scores alike: nothing changes
    got2 = oracle.attention(shape, 0, [0], [n - 1], bt, 2, 5.0 * q, kp, vp)
    np.testing.assert_allclose(got2, got, rtol=1e-12)


def test_attention_gqa_equals_mha_with_duplicated_kv_heads():
    rng = np.random.default_rng(14)
    n_q, n_kv, d, total = 6, 2, 8, 33
    g = n_q // n_kv
    gqa = small_shape(n_q_heads=n_q, n_kv_heads=n_kv, head_dim=d)
    mha = small_shape(n_q_heads=n_q, n_kv_heads=n_q, head_dim=d)
    Kb = bits_of(rng.standard_normal((total, n_kv, d))); Vb = bits_of(rng.standard_normal((total, n_kv, d)))
    bt = np.array([[0, 2, 1]], dtype=np.int32)
    kp, vp = _fill_pool_from_dense(gqa, 3, bt[0], Kb, Vb)
    kp2, vp2 = _fill_pool_from_dense(mha, 3, bt[0], np.repeat(Kb, g, axis=1), np.repeat(Vb, g, axis=1))
    q = rng.standard_normal((total, n_q, d))
    pos = np.arange(total, dtype=np.int32); seq = np.zeros(total, dtype=np.int32)
    a = oracle.attention(gqa, 0, seq, pos, bt, 3, q, kp, vp)
    b = oracle.attention(mha, 0, seq, pos, bt, 3, q, kp2, vp2)
    np.testing.assert_array_equal(a, b)


def test_attention_ignores_positions_after_the_row_and_other_layers():
    shape = small_shape(num_layers=2, n_q_heads=2, n_kv_heads=1, head_dim=8)
    rng = np.random.default_rng(15)
    total, num_pages = 32, 2
    per_layer = synth.pool_elems_per_layer(shape, num_pages)
    Kb = bits_of(rng.standard_normal((total, 1, 8))); Vb = bits_of(rng.standard_normal((total, 1, 8)))
    bt = np.array([[1, 0]], dtype=np.int32)
    k1, v1 = _fill_pool_from_dense(shape, num_pages, bt[0], Kb, Vb)
    junk = bits_of(rng.standard_normal(per_layer))
    kp = np.concatenate([junk, k1]); vp = np.concatenate([junk, v1])     # layer 1 holds the data
    q = rng.standard_normal((1, 2, 8))
    a = oracle.attention(shape, 1, [0], [20], bt, num_pages, q, kp, vp)
    Kb2, Vb2 = Kb.copy(), Vb.copy()
    Kb2[21:] = bits_of(rng.standard_normal((11, 1, 8))); Vb2[21:] = bits_of(rng.standard_normal((11, 1, 8)))
    k2, v2 = _fill_pool_from_dense(shape, num_pages, bt[0], Kb2, Vb2)
    b = oracle.attention(shape, 1, [0], [20], bt, num_pages, q, np.concatenate([k1, k2]), np.concatenate([v1, v2]))
    np.testing.assert_array_equal(a, b)
    want = _brute_force_attention(q, oracle.bf16_to_f64(Kb)[:21], oracle.bf16_to_f64(Vb)[:21], 2, 1, 20)
    np.testing.assert_allclose(a, want, rtol=1e-12)


def test_linear_few_rows_and_many_rows_paths_agree_bitwise():
    """The two loop nests of the linear layer perform the same operations in the same order."""
    rng = np.random.default_rng(16)
    K, N = 96, 600
    x = rng.standard_normal((70, K))
    w = bits_of(rng.standard_normal((N, K)))
    b = bits_of(rng.standard_normal(N))
    many = oracle.linear(x, w, b)               # 70 rows: transposed-copy path
    few = oracle.linear(x[:5], w, b)            # 5 rows: dot-product path
    np.testing.assert_array_equal(few, many[:5])
    one = oracle.linear(x[69:70], w, b)
    np.testing.assert_array_equal(one[0], many[69])
