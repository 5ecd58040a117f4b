"""GPU parity of the whole stage forward (through the C ABI) against the CPU oracle.

Bars: KV slot placement bit-exact (the set of pool elements that change equals the oracle's, every
written value within one bf16 ulp of the oracle's, nothing else touched); stage output within
max abs 2e-2 and sum|d|/sum|ref| 5e-3 of the oracle on the tiny configuration, and, where outputs are
large, within the scale-aware form: y_bf16 == RNE(y_f32) bit-exactly, max|y_f32 - ref| <= 2e-2 max(1, rms(ref)),
sum|y_bf16 - ref| / sum|ref| <= 5e-3.
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2504_14775_amd import binding as B
from paper_2504_14775_amd import synth
from gpu_util import DEV, GpuStage, bits_of, parity_report, to_dev_bits
from helpers import hidden_np, layer_weights_np, pool_np, written_mask

pytestmark = pytest.mark.gpu

SENT = 0x7FC1


def ulp_distance(a_bits, b_bits):
    """Distance in bf16 steps between two finite bf16 bit patterns (sign-magnitude aware)."""
    def key(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7FFF), u & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def check_pool(name, got_bits, before_bits, want_bits, num_layers=1, mask=None):
    """Placement is exact: only the batch's slots change.  Values are held to the output tolerance (the
    library feeds bf16-rounded activations to the matrix cores, the oracle keeps them in double), layer 0
    to one bf16 step at the scale of the values."""
    changed_want = mask if mask is not None else want_bits != before_bits
    assert np.array_equal(want_bits[~changed_want], before_bits[~changed_want]), f"{name}: oracle wrote outside the slots"
    assert np.array_equal(got_bits[~changed_want], before_bits[~changed_want]), f"{name}: wrote outside the batch's slots"
    per_layer = got_bits.size // num_layers
    for l in range(num_layers):
        sl = slice(l * per_layer, (l + 1) * per_layer)
        m = changed_want[sl]
        if not m.any():
            continue
        g, w = got_bits[sl][m], want_bits[sl][m]
        gf, wf = oracle.bf16_to_f64(g), oracle.bf16_to_f64(w)
        assert np.isfinite(gf).all()
        rms = float(np.sqrt((wf ** 2).mean()))
        if l == 0:
            # layer 0: both sides start from the same input; the only difference is the bf16 rounding of the
            # normalised activations feeding the MFMA, worth one to two bf16 steps at the scale of the values
            assert np.all(np.abs(gf - wf) <= 2.0 ** -6 * np.maximum(np.abs(wf), rms)), f"{name}: layer 0 values"
        assert np.abs(gf - wf).max() <= 2e-2 * max(1.0, rms) + 2.0 ** -7 * np.abs(wf).max(), f"{name}: layer {l}"
        assert np.abs(gf - wf).sum() <= 1e-2 * np.abs(wf).sum(), f"{name}: layer {l}"
    return int(changed_want.sum())


def run_both(shape, weights, batch, kp0, vp0, x_bits, stage=None):
    kp, vp = kp0.copy(), vp0.copy()
    ref, ref16 = oracle.stage_forward(shape, weights, batch.new_tokens, batch.cached_len, batch.block_tables,
                                      batch.num_blocks, kp, vp, x_bits)
    stage = stage or GpuStage(shape, weights, [batch])
    dk, dv = to_dev_bits(kp0), to_dev_bits(vp0)
    out, out32 = stage.run(batch, dk, dv, to_dev_bits(x_bits))
    return dict(ref=ref, ref16=ref16, kp=kp, vp=vp, out=bits_of(out), out32=out32.cpu().numpy(),
                gk=bits_of(dk), gv=bits_of(dv), stage=stage)


def assert_output(name, r, literal):
    rep = parity_report(name, r["out"], r["out32"], r["ref"])
    # (i) the bf16 output is the fp32 residual stream rounded to nearest even
    assert np.array_equal(r["out"], bits_of(torch.from_numpy(r["out32"]).to(torch.bfloat16)))
    if literal:
        assert rep["max_abs_bf16"] <= 2e-2
    assert rep["max_abs_f32_scaled"] <= 2e-2
    assert rep["mean_rel_bf16"] <= 5e-3
    return rep


def test_tiny_configuration_full_parity():
    print("tiny configuration, seed 0", flush=True)
    shape = synth.SHAPES["tiny"]
    batch = synth.make_batch("tiny", 0)
    w = layer_weights_np(shape, 0)
    kp0, vp0 = pool_np(shape, 0, batch.num_blocks)
    r = run_both(shape, w, batch, kp0, vp0, hidden_np(shape, 0, batch.num_tokens))
    assert_output("tiny", r, literal=True)
    mk, mv = written_mask(shape, batch)
    n = check_pool("K", r["gk"], kp0, r["kp"], mask=mk)
    check_pool("V", r["gv"], vp0, r["vp"], mask=mv)
    assert n == batch.num_tokens * shape.n_kv_heads * shape.head_dim


def test_tiny_slot_placement_with_sentinel_pool():
    print("tiny configuration, sentinel pool for decode prefixes filled by a first pass", flush=True)
    shape = synth.SHAPES["tiny"]
    w = layer_weights_np(shape, 0)
    # pass 1 prefills every sequence up to its cached length into a sentinel pool, pass 2 is the tiny batch
    batch = synth.make_batch("tiny", 0)
    pre = [(int(c), 0) for c in batch.cached_len if c > 0]
    idx = [i for i, c in enumerate(batch.cached_len) if c > 0]
    b1 = synth.Batch(np.array([n for n, _ in pre], dtype=np.int32), np.zeros(len(pre), dtype=np.int32),
                     batch.block_tables[idx].copy(), batch.num_blocks)
    n_el = shape.num_layers * synth.pool_elems_per_layer(shape, batch.num_blocks)
    kp0 = np.full(n_el, SENT, dtype=np.uint16); vp0 = kp0.copy()
    x1 = hidden_np(shape, 11, b1.num_tokens)
    stage = GpuStage(shape, w, [batch, b1])
    r1 = run_both(shape, w, b1, kp0, vp0, x1, stage)
    changed = check_pool("K pass1", r1["gk"], kp0, r1["kp"])
    check_pool("V pass1", r1["gv"], vp0, r1["vp"])
    assert changed == b1.num_tokens * shape.n_kv_heads * shape.head_dim * shape.num_layers
    # pass 2 continues from the oracle's pool image (identical inputs for both sides)
    r2 = run_both(shape, w, batch, r1["kp"], r1["vp"], hidden_np(shape, 0, batch.num_tokens), stage)
    check_pool("K pass2", r2["gk"], r1["kp"], r2["kp"])
    check_pool("V pass2", r2["gv"], r1["vp"], r2["vp"])
    assert_output("tiny-after-prefill", r2, literal=True)


def test_page_permutation_is_bitwise_invisible_and_runs_are_deterministic():
    print("page permutation + determinism on the tiny configuration", flush=True)
    shape = synth.SHAPES["tiny"]
    batch = synth.make_batch("tiny", 0)
    w = layer_weights_np(shape, 0)
    kp0, vp0 = pool_np(shape, 0, batch.num_blocks)
    x = to_dev_bits(hidden_np(shape, 0, batch.num_tokens))
    stage = GpuStage(shape, w, [batch])
    a, a32 = stage.run(batch, to_dev_bits(kp0), to_dev_bits(vp0), x)
    a2, _ = stage.run(batch, to_dev_bits(kp0), to_dev_bits(vp0), x)
    assert torch.equal(a.view(torch.int16), a2.view(torch.int16))
    perm = np.random.default_rng(5).permutation(batch.num_blocks)
    bt2 = np.where(batch.block_tables >= 0, perm[np.clip(batch.block_tables, 0, None)], -1).astype(np.int32)
    per_page = shape.n_kv_heads * shape.page_size * shape.head_dim
    k2 = np.empty_like(kp0); v2 = np.empty_like(vp0)
    k2.reshape(shape.num_layers, -1, per_page)[:, perm, :] = kp0.reshape(shape.num_layers, -1, per_page)
    v2.reshape(shape.num_layers, -1, per_page)[:, perm, :] = vp0.reshape(shape.num_layers, -1, per_page)
    b2 = dataclasses.replace(batch, block_tables=bt2)
    b, b32 = stage.run(b2, to_dev_bits(k2), to_dev_bits(v2), x)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert torch.equal(a32, b32)


MID = synth.StageShape("mid", 3, 512, 16, 2, 128, 1032)


def mid_batch(seed):
    seqs = [(150, 70), (64, 0), (2, 300), (1, 0), (1, 1), (1, 15), (1, 16), (1, 255), (1, 256), (1, 257),
            (1, 700), (1, 1500), (33, 31)]
    return synth.build_batch(seqs, seed, spare_blocks=9, label="mid")


def test_mid_shape_multi_layer_ragged_batch():
    """d=128, 8 query heads per KV head, 3 layers, lengths that straddle page, block and partition edges."""
    print("mid shape ragged batch", flush=True)
    batch = mid_batch(4)
    w = layer_weights_np(MID, 4)
    kp0, vp0 = pool_np(MID, 4, batch.num_blocks)
    r = run_both(MID, w, batch, kp0, vp0, hidden_np(MID, 4, batch.num_tokens))
    assert_output("mid", r, literal=False)
    mk, mv = written_mask(MID, batch)
    check_pool("K", r["gk"], kp0, r["kp"], MID.num_layers, mask=mk)
    check_pool("V", r["gv"], vp0, r["vp"], MID.num_layers, mask=mv)


@pytest.mark.parametrize("min_wgs", [1, 64, 10 ** 6])
def test_decode_rows_whole_or_partitioned_match_the_oracle(min_wgs):
    """decode_min_workgroups = 1 leaves every decode row whole (finished by the attention kernel itself);
    10^6 cuts rows down to the smallest partition (256 keys) and sends them through the merge kernel; 64 mixes
    both in one batch.  All three must meet the oracle and agree with each other to fp32 rounding."""
    print(f"decode partitioning, decode_min_workgroups={min_wgs}", flush=True)
    one_layer = dataclasses.replace(MID, num_layers=1, name="mid1")
    seqs = [(1, 0), (1, 31), (1, 32), (1, 255), (1, 256), (1, 257), (1, 511), (1, 512), (1, 700), (1, 1023),
            (1, 1500), (40, 9)]
    batch = synth.build_batch(seqs, 11, spare_blocks=5, label="dec")
    w = layer_weights_np(one_layer, 11)
    kp0, vp0 = pool_np(one_layer, 11, batch.num_blocks)
    x = hidden_np(one_layer, 11, batch.num_tokens)
    stage = GpuStage(one_layer, w, [batch])
    stage.stage.set_option("decode_min_workgroups", min_wgs)
    r = run_both(one_layer, w, batch, kp0, vp0, x, stage=stage)
    assert_output(f"dec{min_wgs}", r, literal=False)
    base = GpuStage(one_layer, w, [batch])
    _, base32 = base.run(batch, to_dev_bits(kp0), to_dev_bits(vp0), to_dev_bits(x))
    rms = float(np.sqrt((r["ref"] ** 2).mean()))
    assert np.abs(r["out32"] - base32.cpu().numpy()).max() <= 1e-3 * max(1.0, rms)


def test_qkv_bias_and_nan_sentinels_in_unused_slots():
    print("qkv bias + NaN sentinel in never-written slots", flush=True)
    shape = dataclasses.replace(synth.SHAPES["tiny"], has_qkv_bias=True, name="tiny_bias")
    batch = synth.build_batch([(21, 0), (5, 0), (1, 0)], 6, spare_blocks=3)
    w = layer_weights_np(shape, 6)
    n_el = shape.num_layers * synth.pool_elems_per_layer(shape, batch.num_blocks)
    kp0 = np.full(n_el, SENT, dtype=np.uint16); vp0 = kp0.copy()      # NaN bit pattern everywhere
    r = run_both(shape, w, batch, kp0, vp0, hidden_np(shape, 6, batch.num_tokens))
    assert np.isfinite(r["out32"]).all()
    assert_output("bias", r, literal=True)
    check_pool("K", r["gk"], kp0, r["kp"])
    check_pool("V", r["gv"], vp0, r["vp"])


def test_chunked_and_decode_invariants_on_gpu():
    print("chunked == unchunked and decode == last causal row on the GPU (within tolerance)", flush=True)
    shape = dataclasses.replace(synth.SHAPES["tiny"], num_layers=2, name="tiny2")
    w = layer_weights_np(shape, 8)
    total = 80
    full = synth.build_batch([(total, 0)], 8, spare_blocks=2)
    x = hidden_np(shape, 8, total)
    n_el = shape.num_layers * synth.pool_elems_per_layer(shape, full.num_blocks)
    blank = np.full(n_el, SENT, dtype=np.uint16)
    stage = GpuStage(shape, w, [full])
    dk, dv = to_dev_bits(blank), to_dev_bits(blank)
    ref_out, ref32 = stage.run(full, dk, dv, to_dev_bits(x))
    ref_k = bits_of(dk)
    dk2, dv2 = to_dev_bits(blank), to_dev_bits(blank)
    outs = []
    done = 0
    for n in (48, 31, 1):
        b = synth.Batch(np.array([n], dtype=np.int32), np.array([done], dtype=np.int32), full.block_tables,
                        full.num_blocks)
        o, o32 = stage.run(b, dk2, dv2, to_dev_bits(x[done:done + n]))
        outs.append(o32.cpu().numpy())
        done += n
    got = np.concatenate(outs)
    want = ref32.cpu().numpy()
    rms = float(np.sqrt((want.astype(np.float64) ** 2).mean()))
    assert np.abs(got - want).max() <= 2e-2 * max(1.0, rms)
    per_layer = ref_k.size // shape.num_layers
    assert np.array_equal(bits_of(dk2)[:per_layer], ref_k[:per_layer])   # a row's K does not depend on the batch


def test_forward_rejects_malformed_batches_without_side_effects():
    print("error paths", flush=True)
    shape = synth.SHAPES["tiny"]
    batch = synth.make_batch("tiny", 0)
    w = layer_weights_np(shape, 0)
    kp0, vp0 = pool_np(shape, 0, batch.num_blocks)
    stage = GpuStage(shape, w, [batch])
    dk, dv = to_dev_bits(kp0), to_dev_bits(vp0)
    x = to_dev_bits(hidden_np(shape, 0, batch.num_tokens))
    out = torch.zeros(batch.num_tokens, shape.hidden, dtype=torch.bfloat16, device=DEV)
    st = stage.stage
    st.bind_kv_pool(dk, dv, batch.num_blocks)

    def status_of(nt, cl, bt):
        try:
            st.forward(nt, cl, bt, x, out)
        except B.GllmError as e:
            return e.status
        return 0

    nt, cl, bt = batch.new_tokens.copy(), batch.cached_len.copy(), batch.block_tables.copy()
    bad = nt.copy(); bad[2] = 0
    assert status_of(bad, cl, bt) == -1
    bad = cl.copy(); bad[0] = -1
    assert status_of(nt, bad, bt) == -1
    bad = bt.copy(); bad[0, 0] = batch.num_blocks
    assert status_of(nt, cl, bad) == -3
    bad = bt.copy(); bad[2, 1] = bt[3, 1]          # two decode rows write into the same physical page
    assert status_of(nt, cl, bad) == -4
    bad = cl.copy(); bad[5] = 4000
    assert status_of(nt, bad, bt) == -2
    big = np.concatenate([nt, nt]); bigc = np.concatenate([cl, cl]); bigb = np.concatenate([bt, bt])
    assert status_of(big, bigc, bigb) in (-1, -2)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(dk), kp0) and np.array_equal(bits_of(dv), vp0)
    assert int(out.view(torch.int16).abs().sum()) == 0
    assert "share a physical page" in st.last_error() or st.last_error()
    # a stage without pool / weights refuses to run
    fresh = B.stage_for_batches(shape, [batch])
    with pytest.raises(B.GllmError) as e:
        fresh.forward(nt, cl, bt, x, out)
    assert e.value.status == -5
    assert status_of(nt, cl, bt) == 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("n_q,n_kv,d", [(6, 2, 128), (4, 4, 64), (8, 2, 64), (8, 1, 128), (10, 2, 64), (2, 1, 128)])
def test_head_group_shapes(n_q, n_kv, d):
    """Every query-heads-per-KV-head case of the attention kernels (1, 2, 3, 4, 5, 8) at both head sizes, on a
    batch whose chunks span several 32-key blocks, item boundaries and ragged tails."""
    print(f"head grouping n_q={n_q} n_kv={n_kv} d={d}", flush=True)
    shape = synth.StageShape("grp", 2, 256, n_q, n_kv, d, 384)
    seqs = [(150, 37), (130, 0), (1, 99), (1, 0), (17, 200), (1, 511), (3, 30)]
    batch = synth.build_batch(seqs, 9, spare_blocks=5)
    w = layer_weights_np(shape, 9)
    kp0, vp0 = pool_np(shape, 9, batch.num_blocks)
    r = run_both(shape, w, batch, kp0, vp0, hidden_np(shape, 9, batch.num_tokens))
    assert_output(f"grp{n_q}/{n_kv}/{d}", r, literal=False)
    mk, mv = written_mask(shape, batch)
    check_pool("K", r["gk"], kp0, r["kp"], shape.num_layers, mask=mk)
    check_pool("V", r["gv"], vp0, r["vp"], shape.num_layers, mask=mv)


def test_two_stage_objects_over_one_set_of_weights():
    """A stage that borrows another's weights gives bit-identical outputs and pools, refuses weights of its own
    afterwards, and refuses an owner of another shape or one that is not fully loaded."""
    print("shared weights", flush=True)
    shape = dataclasses.replace(synth.SHAPES["tiny"], num_layers=2, name="tiny_two_layers")
    batch = synth.make_batch("tiny", 4)
    w = layer_weights_np(shape, 4)
    kp0, vp0 = pool_np(shape, 4, batch.num_blocks)
    x = to_dev_bits(hidden_np(shape, 4, batch.num_tokens))
    owner = GpuStage(shape, w, [batch])
    borrower = B.stage_for_batches(shape, [batch])
    other = B.stage_for_batches(dataclasses.replace(shape, intermediate=shape.intermediate + 128), [batch])
    unloaded = B.stage_for_batches(shape, [batch])
    for bad, code in ((other, -1), (unloaded, -5), (borrower, -1)):
        with pytest.raises(B.GllmError) as e:
            borrower.share_weights(bad)
        assert e.value.status == code, borrower.last_error()
    borrower.share_weights(owner.stage)
    with pytest.raises(B.GllmError) as e:
        unloaded.share_weights(borrower)                      # no chains of borrowers
    assert e.value.status == -1
    with pytest.raises(B.GllmError) as e:
        borrower.load_layer(0, {k: to_dev_bits(v) for k, v in w[0].items()})
    assert e.value.status == -5
    got = []
    for st in (owner.stage, borrower):
        dk, dv = to_dev_bits(kp0), to_dev_bits(vp0)
        out = torch.empty(batch.num_tokens, shape.hidden, dtype=torch.bfloat16, device=DEV)
        st.bind_kv_pool(dk, dv, batch.num_blocks)
        st.forward(batch.new_tokens, batch.cached_len, batch.block_tables, x, out)
        torch.cuda.synchronize()
        got.append((bits_of(out), bits_of(dk), bits_of(dv)))
    for a, b in zip(*got):
        assert np.array_equal(a, b)
    borrower.destroy()                                        # must leave the owner's buffers alone
    dk, dv = to_dev_bits(kp0), to_dev_bits(vp0)
    out, _ = owner.run(batch, dk, dv, x, want_f32=False)
    assert np.array_equal(bits_of(out), got[0][0])


def sentinel_pool_with_prefixes(shape, batch, seed):
    """A pool of sentinel bit patterns in which only the cached positions of the batch's sequences hold real values
    (the generator's): what a forward pass may read is defined, everything it must not touch is recognisable."""
    n_el = shape.num_layers * synth.pool_elems_per_layer(shape, batch.num_blocks)
    kp0 = np.full(n_el, SENT, dtype=np.uint16)
    vp0 = kp0.copy()
    kg, vg = pool_np(shape, seed, batch.num_blocks)
    cached = np.zeros((batch.num_blocks, 16), dtype=bool)
    for s in range(batch.num_seqs):
        pos = np.arange(int(batch.cached_len[s]))
        cached[batch.block_tables[s, pos // 16], pos % 16] = True
    L, nkv, d = shape.num_layers, shape.n_kv_heads, shape.head_dim
    km = np.broadcast_to(cached[None, :, None, None, :, None], (L, batch.num_blocks, nkv, d // 8, 16, 8)).reshape(-1)
    vm = np.broadcast_to(cached[None, :, None, None, :], (L, batch.num_blocks, nkv, d, 16)).reshape(-1)
    kp0[km], vp0[vm] = kg[km], vg[vm]
    return kp0, vp0


@pytest.mark.parametrize("hidden,planes", [(256, 1), (1024, 2)])
def test_chunk_runs_at_every_page_alignment_write_exactly_their_slots(hidden, planes):
    """Chunks whose tokens fall into pages in every way the V writer distinguishes: a run that ends a page, one that
    starts one, whole pages, a run of one at either edge, a chunk inside a single page, next to decode rows.  The pool
    starts as a sentinel pattern: exactly the slots of the new tokens change, and they hold the oracle's values.
    (The hidden size decides whether the QKV projection is split along k: the single-plane writer and the general one.)"""
    print(f"chunk runs vs page boundaries, hidden {hidden}: {planes} plane(s)", flush=True)
    shape = synth.StageShape("runs", 1, hidden, 4, 2, 64, 384)
    #        (new, cached): 15|16 split    one page    page+1      1+page+1     inside    decode rows
    seqs = [(2, 15), (16, 16), (17, 32), (18, 15), (5, 3), (1, 15), (1, 16), (1, 0), (33, 0), (31, 17)]
    batch = synth.build_batch(seqs, 21, spare_blocks=3)
    assert B.gllm_op_gemm_plan(batch.num_tokens, 512, hidden, 0, 8)[1] == planes
    w = layer_weights_np(shape, 21)
    kp0, vp0 = sentinel_pool_with_prefixes(shape, batch, 21)
    r = run_both(shape, w, batch, kp0, vp0, hidden_np(shape, 21, batch.num_tokens))
    assert_output("runs", r, literal=False)
    mk, mv = written_mask(shape, batch)
    n = check_pool("K", r["gk"], kp0, r["kp"], mask=mk)
    check_pool("V", r["gv"], vp0, r["vp"], mask=mv)
    assert n == batch.num_tokens * shape.n_kv_heads * shape.head_dim


def test_random_ragged_batches_match_the_oracle():
    """Twenty seeded random hybrid batches on a small two-layer shape -- decode rows, chunks of every length up to a
    few pages at arbitrary cached lengths, in arbitrary order -- against the oracle: output within the tolerance,
    exactly the new tokens' slots written."""
    shape = synth.StageShape("ragged", 2, 256, 8, 2, 64, 384)
    w = layer_weights_np(shape, 33)
    rng = np.random.default_rng(33)
    sizing = synth.build_batch([(70, 130)] * 10, 1)
    stage = GpuStage(shape, w, [sizing])
    for case in range(20):
        n_seq = int(rng.integers(1, 11))
        seqs = []
        for _ in range(n_seq):
            new = 1 if rng.random() < 0.55 else int(rng.integers(2, 71))
            seqs.append((new, int(rng.integers(0, 131))))
        print(f"random batch {case}: {seqs}", flush=True)
        batch = synth.build_batch(seqs, 100 + case, spare_blocks=int(rng.integers(0, 4)), max_blocks_per_seq=sizing.block_tables.shape[1])
        kp0, vp0 = sentinel_pool_with_prefixes(shape, batch, 100 + case)
        r = run_both(shape, w, batch, kp0, vp0, hidden_np(shape, 100 + case, batch.num_tokens), stage)
        assert_output(f"ragged{case}", r, literal=False)
        mk, mv = written_mask(shape, batch)
        check_pool("K", r["gk"], kp0, r["kp"], shape.num_layers, mask=mk)
        check_pool("V", r["gv"], vp0, r["vp"], shape.num_layers, mask=mv)


def test_layer_range_option_runs_a_part_of_the_stage():
    """layer_begin / layer_end: layers [0, l) equal an l-layer stage of the same weights bit for bit; layer l alone
    equals a one-layer stage holding layer l's weights over layer l's slice of the pool, bit for bit, pool included;
    layers outside the range leave their pool slices alone."""
    print("layer range option, 3-layer stage", flush=True)
    shape = dataclasses.replace(synth.SHAPES["tiny"], num_layers=3)
    batch = synth.make_batch("tiny", 0)
    w = layer_weights_np(shape, 4)
    kp0, vp0 = pool_np(shape, 4, batch.num_blocks)
    x = to_dev_bits(hidden_np(shape, 4, batch.num_tokens))
    per_layer = synth.pool_elems_per_layer(shape, batch.num_blocks)
    whole = GpuStage(shape, w, [batch])
    for l in (1, 2):
        dk, dv = to_dev_bits(kp0), to_dev_bits(vp0)
        whole.stage.set_option("layer_begin", 0)
        whole.stage.set_option("layer_end", l)
        head, head32 = whole.run(batch, dk, dv, x)
        short = GpuStage(dataclasses.replace(shape, num_layers=l), w[:l], [batch])
        sk, sv = to_dev_bits(kp0[:l * per_layer]), to_dev_bits(vp0[:l * per_layer])
        want, want32 = short.run(batch, sk, sv, x)
        assert torch.equal(head.view(torch.int16), want.view(torch.int16)) and torch.equal(head32, want32)
        assert np.array_equal(bits_of(dk)[:l * per_layer], bits_of(sk)) and np.array_equal(bits_of(dv)[:l * per_layer], bits_of(sv))
        assert np.array_equal(bits_of(dk)[l * per_layer:], kp0[l * per_layer:])        # later layers untouched
        short.stage.destroy()
        # layer l alone, fed the bf16 output of the layers before it
        whole.stage.set_option("layer_begin", l)          # moves layer_end to l + 1
        whole.stage.set_option("layer_end", l + 1)
        dk2, dv2 = to_dev_bits(kp0), to_dev_bits(vp0)
        tail, tail32 = whole.run(batch, dk2, dv2, head)
        one = GpuStage(dataclasses.replace(shape, num_layers=1), [w[l]], [batch])
        ok, ov = to_dev_bits(kp0[l * per_layer:(l + 1) * per_layer]), to_dev_bits(vp0[l * per_layer:(l + 1) * per_layer])
        want, want32 = one.run(batch, ok, ov, head)
        assert torch.equal(tail.view(torch.int16), want.view(torch.int16)) and torch.equal(tail32, want32)
        assert np.array_equal(bits_of(dk2)[l * per_layer:(l + 1) * per_layer], bits_of(ok))
        assert np.array_equal(bits_of(dk2)[:l * per_layer], kp0[:l * per_layer])
        one.stage.destroy()
    for name, v in (("layer_begin", -1), ("layer_begin", 3), ("layer_end", 0), ("layer_end", 4)):
        with pytest.raises(B.GllmError):
            whole.stage.set_option(name, v)
    whole.stage.destroy()


def test_row_mixed_option_belongs_to_one_stage():
    """Two stage objects: switching gemm_row_mixed off on one must not change what the other computes or how."""
    shape = synth.SHAPES["tiny"]
    batch = synth.build_batch([(300, 0)], 0, label="300 rows")      # 300 rows: a band of 256 plus a short one
    w = layer_weights_np(shape, 5)
    kp0, vp0 = pool_np(shape, 5, batch.num_blocks)
    x = to_dev_bits(hidden_np(shape, 5, batch.num_tokens))
    a, b = GpuStage(shape, w, [batch]), GpuStage(shape, w, [batch])
    ref_a = a.run(batch, to_dev_bits(kp0), to_dev_bits(vp0), x)[1]
    b.stage.set_option("gemm_row_mixed", 0)
    out_b = b.run(batch, to_dev_bits(kp0), to_dev_bits(vp0), x)[1]
    out_a = a.run(batch, to_dev_bits(kp0), to_dev_bits(vp0), x)[1]
    assert torch.equal(out_a, ref_a)                                    # a's plan is unchanged
    assert torch.allclose(out_a, out_b, rtol=0, atol=5e-3)              # same result either way (tile shapes and split counts may differ)
    a.stage.destroy(); b.stage.destroy()


def test_empty_batch_and_batches_at_the_stage_limits():
    """Degenerate and extreme batches: no sequences at all (nothing is enqueued, nothing changes); one token on its own
    (first token of a sequence: attends to itself only, so the attention output is its own V); a batch that uses every
    row, every sequence and the last position the stage was created for; one more of any of them is refused."""
    print("empty batch and limits", flush=True)
    shape = synth.SHAPES["tiny"]
    w = layer_weights_np(shape, 6)
    limit = synth.build_batch([(40, 88), (1, 127), (23, 0)], 6, spare_blocks=2)      # 64 rows, 3 sequences, positions up to 128
    cfg = B.make_config(shape, 64, 3, 8, 128)
    st = B.Stage(cfg)
    ws = torch.empty(st.workspace_bytes(), dtype=torch.uint8, device=DEV)
    st.bind_workspace(ws)
    for l, lw in enumerate(w):
        st.load_layer(l, {k: to_dev_bits(v) for k, v in lw.items()})
    kp0, vp0 = pool_np(shape, 6, limit.num_blocks)
    dk, dv = to_dev_bits(kp0), to_dev_bits(vp0)
    st.bind_kv_pool(dk, dv, limit.num_blocks)
    x = hidden_np(shape, 6, 64)
    out = torch.zeros(64, shape.hidden, dtype=torch.bfloat16, device=DEV)
    # no sequences
    st.forward(np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros((0, 8), np.int32), to_dev_bits(x), out)
    torch.cuda.synchronize()
    assert int(out.view(torch.int16).abs().sum()) == 0
    assert np.array_equal(bits_of(dk), kp0) and np.array_equal(bits_of(dv), vp0)
    # exactly at the limits: against the oracle
    kp, vp = kp0.copy(), vp0.copy()
    ref, _ = oracle.stage_forward(shape, w, limit.new_tokens, limit.cached_len, limit.block_tables, limit.num_blocks, kp, vp, x)
    out32 = torch.empty(64, shape.hidden, dtype=torch.float32, device=DEV)
    st.forward(limit.new_tokens, limit.cached_len, limit.block_tables, to_dev_bits(x), out, out32)
    torch.cuda.synchronize()
    r = dict(ref=ref, out=bits_of(out), out32=out32.cpu().numpy())
    assert_output("limits", r, literal=True)
    mk, mv = written_mask(shape, limit)
    check_pool("K", bits_of(dk), kp0, kp, mask=mk)
    check_pool("V", bits_of(dv), vp0, vp, mask=mv)
    # one past each limit
    def status_of(nt, cl, bt):
        try:
            st.forward(np.asarray(nt, np.int32), np.asarray(cl, np.int32), bt, to_dev_bits(x), out)
        except B.GllmError as e:
            return e.status
        return 0
    bt = limit.block_tables
    assert status_of([41, 1, 23], limit.cached_len, bt) == -2                   # 65 rows
    assert status_of([40, 1, 23], [88, 128, 0], bt) == -2                       # position 129
    four = np.concatenate([bt, bt[:1]])
    assert status_of([40, 1, 22, 1], [88, 127, 0, 0], four) == -1               # a fourth sequence
    # a single first token: softmax over one key
    one = synth.build_batch([(1, 0)], 7)
    kp1, vp1 = pool_np(shape, 7, one.num_blocks)
    d1k, d1v = to_dev_bits(kp1), to_dev_bits(vp1)
    st.bind_kv_pool(d1k, d1v, one.num_blocks)
    k1, v1 = kp1.copy(), vp1.copy()
    ref1, _ = oracle.stage_forward(shape, w, one.new_tokens, one.cached_len, one.block_tables, one.num_blocks, k1, v1, x[:1])
    o1 = torch.empty(1, shape.hidden, dtype=torch.bfloat16, device=DEV); o132 = torch.empty(1, shape.hidden, dtype=torch.float32, device=DEV)
    bt1 = np.full((1, 8), -1, np.int32); bt1[0, 0] = one.block_tables[0, 0]
    st.forward(one.new_tokens, one.cached_len, bt1, to_dev_bits(x[:1]), o1, o132)
    torch.cuda.synchronize()
    assert_output("one token", dict(ref=ref1, out=bits_of(o1), out32=o132.cpu().numpy()), literal=True)
    st.destroy()
