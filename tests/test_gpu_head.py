"""GPU parity of the first / last stage extras (include/gllm_head.h) against oracle/head_oracle.py.

Bars: the embedding is a copy (bit-exact); logits within the stage's tolerance (max abs 2e-2, sum|d|/sum|ref| 5e-3:
the only difference is the bf16 rounding of the normalised hidden state in front of the matrix cores); greedy
tokens exact.  Sampled tokens are decided by fp32 sums on the GPU and float64 sums in the oracle, so a draw whose
u lands within rounding of a boundary may legitimately fall to the neighbouring token: every GPU token must be a
kept token whose interval of the running sum contains u within 1e-4, and nearly all must equal the oracle's.
"""
import numpy as np
import pytest
import torch

from oracle import head_oracle as Hd
from paper_2504_14775_amd import binding as B
from paper_2504_14775_amd import head as HD
from paper_2504_14775_amd import synth
from gpu_util import DEV, bits_of, to_dev_bits

pytestmark = pytest.mark.gpu


def bf16_bits_normal(seed, stream, n, scale, mean=0.0):
    return synth.bf16_bits(synth.normal_bf16(seed, stream, 0, n, scale, mean))


def test_embedding_is_a_row_copy():
    print("embedding", flush=True)
    V, H, T = 777, 256, 300
    table = bf16_bits_normal(1, 1, V * H, 1.0).reshape(V, H)
    rng = np.random.default_rng(0)
    ids = rng.integers(0, V, size=T).astype(np.int32)
    ids[[3, 50, 299]] = [-1, V, 2 ** 30]
    out = torch.full((T, H + 64), 7.0, dtype=torch.bfloat16, device=DEV)[:, :H + 64]
    HD.gllm_op_embedding(torch.from_numpy(ids).to(DEV), to_dev_bits(table), out)
    torch.cuda.synchronize()
    got = bits_of(out)
    assert np.array_equal(got[:, :H], Hd.embedding(table, ids))
    assert np.all(got[:, H:] == bits_of(torch.tensor([7.0], dtype=torch.bfloat16))[0])      # nothing past a row's hidden size


@pytest.mark.parametrize("H,V,T,M,sample_cols", [(256, 1000, 50, 17, None), (4096, 128256, 300, 64, 1500), (5120, 152064, 8, 3, 1500)])
def test_logits_match_the_oracle(H, V, T, M, sample_cols):
    print(f"logits H={H} V={V} rows={M}", flush=True)
    eps = 1e-6
    gain = bf16_bits_normal(2, 1, H, 0.1, 1.0)
    w = synth.normal_bf16(2, 2, 0, V * H, 0.02, 0.0, device=DEV).view(V, H)
    x = (torch.randn(T, H, generator=torch.Generator().manual_seed(3)) * 3.0).to(torch.float32)
    rng = np.random.default_rng(4)
    rows = rng.integers(0, T, size=M).astype(np.int32)
    rows[0] = rows[-1]                                                    # a repeated row is allowed
    head = HD.Head(H, V, max(M, 4), eps)
    head.load(to_dev_bits(gain), w)
    out = torch.full((M, head.padded_vocab), float("nan"), dtype=torch.float32, device=DEV)
    head.logits(x.to(DEV), torch.from_numpy(rows).to(DEV), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert head.padded_vocab % 256 == 0 and head.padded_vocab >= V
    assert not np.isnan(got).any() and not got[:, V:].any()               # padding columns are written as zeros
    cols = np.arange(V) if sample_cols is None else np.sort(rng.choice(V, size=sample_cols, replace=False))
    w_bits = synth.bf16_bits(w[torch.from_numpy(cols).to(DEV)].cpu())
    ref = Hd.final_logits(x.numpy().astype(np.float64), rows, gain, w_bits, eps)
    d = np.abs(got[:, cols] - ref)
    print(f"[parity] logits: max_abs={d.max():.4g} mean_rel={d.sum() / np.abs(ref).sum():.4g} rms_ref={np.sqrt((ref ** 2).mean()):.3g}", flush=True)
    assert d.max() <= 2e-2 and d.sum() / np.abs(ref).sum() <= 5e-3
    with pytest.raises(B.GllmError) as e:
        head.logits(x.to(DEV), torch.zeros(max(M, 4) + 1, dtype=torch.int32, device=DEV),
                    torch.empty(max(M, 4) + 1, head.padded_vocab, dtype=torch.float32, device=DEV))
    assert e.value.status == -2
    head.destroy()


def test_head_refuses_use_before_load_and_bad_arguments():
    head = HD.Head(256, 100, 4, 1e-6)
    x = torch.zeros(4, 256, device=DEV)
    rows = torch.zeros(2, dtype=torch.int32, device=DEV)
    with pytest.raises(B.GllmError) as e:
        head.logits(x, rows, torch.empty(2, 256, device=DEV))
    assert e.value.status == -5
    head.load(torch.ones(256, dtype=torch.bfloat16, device=DEV), torch.zeros(100, 256, dtype=torch.bfloat16, device=DEV))
    with pytest.raises(B.GllmError) as e:
        head.logits(x, rows, torch.empty(2, 128, device=DEV))             # narrower than the padded vocabulary
    assert e.value.status == -1
    for bad in ((100, 100, 4), (256, 0, 4), (256, 100, 0)):
        with pytest.raises(B.GllmError):
            HD.Head(*bad, 1e-6)
    head.destroy()


def run_sampler(logits, V, temp, k, p, u):
    M = logits.shape[0]
    out = torch.full((M,), -7, dtype=torch.int32, device=DEV)
    HD.gllm_op_sample(logits, V, torch.tensor(temp, dtype=torch.float32, device=DEV), torch.tensor(k, dtype=torch.int32, device=DEV),
                      torch.tensor(p, dtype=torch.float32, device=DEV), torch.tensor(u, dtype=torch.float32, device=DEV), out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_greedy_and_its_equivalents_are_exact():
    print("sampler: greedy", flush=True)
    V, M = 5000, 12
    lg = torch.randn(M, V + 24, generator=torch.Generator().manual_seed(5)) * 2.0
    lg[:, V:] = 100.0                                                     # columns past the vocabulary must be ignored
    lg[1, 17] = lg[1, 4000] = lg[1].max() + 1.0                           # a tie: the lower index wins
    lg[2, 0] = 50.0
    lg[3, V - 1] = 50.0
    ref = np.array([Hd.greedy(lg[i, :V].numpy()) for i in range(M)])
    assert ref[1] == 17 and ref[2] == 0 and ref[3] == V - 1
    d = lg.to(DEV)
    u = [0.0, 0.5, 0.999] * 4
    assert np.array_equal(run_sampler(d, V, [0.0] * M, [0] * M, [1.0] * M, u), ref)
    assert np.array_equal(run_sampler(d, V, [-1.0] * M, [5] * M, [0.3] * M, u), ref)
    got = run_sampler(d, V, [1.0] * M, [1] * M, [1.0] * M, u)                 # top-1 (row 1 keeps both tied tokens)
    assert np.array_equal(np.delete(got, 1), np.delete(ref, 1)) and got[1] in (17, 4000)
    got = run_sampler(d, V, [0.7] * M, [0] * M, [1e-6] * M, u)                # a vanishing nucleus
    assert np.array_equal(np.delete(got, 1), np.delete(ref, 1)) and got[1] in (17, 4000)


def check_against_oracle(lg, temp, k, p, u, label, slack=2):
    """lg: float32 [M, V] on the host.  Every GPU token must be a kept token whose interval of the running sum
    contains u within 1e-4; all but `slack` must equal the oracle's."""
    M, V = lg.shape
    got = run_sampler(lg.to(DEV), V, temp.tolist(), k.tolist(), p.tolist(), u.tolist())
    same = 0
    for i in range(M):
        row = lg[i].numpy()
        want = Hd.sample(row, float(temp[i]), int(k[i]), float(p[i]), float(u[i]))
        keep, prob = Hd.kept_distribution(row, float(temp[i]), int(k[i]), float(p[i]))
        gi = int(got[i])
        assert 0 <= gi < V, (i, gi)
        if gi == want:
            same += 1
            continue
        cum = np.cumsum(prob)
        lo = cum[gi] - prob[gi]
        assert keep[gi] and lo - 1e-4 <= float(u[i]) <= cum[gi] + 1e-4, (i, gi, want, float(u[i]), lo, cum[gi])
    print(f"[parity] sampler {label}: {same}/{M} tokens equal the oracle's", flush=True)
    assert same >= M - slack


@pytest.mark.parametrize("V,M,scale", [(1000, 48, 2.0), (1003, 48, 2.0), (5000, 48, 3.0), (152064, 24, 2.5)])   # 1003: rows off the 16-byte grid, and a tail
def test_sampled_tokens_follow_the_oracle(V, M, scale):
    print(f"sampler: V={V} rows={M}", flush=True)
    g = torch.Generator().manual_seed(V)
    lg = (torch.randn(M, V, generator=g) * scale).to(torch.float32)
    rng = np.random.default_rng(V)
    temp = rng.choice([0.5, 0.8, 1.0, 1.3], size=M).astype(np.float32)
    k = rng.choice([0, 1, 2, 10, 50, V // 2, V, V + 5], size=M).astype(np.int32)
    p = rng.choice([1.0, 0.95, 0.9, 0.5, 0.1], size=M).astype(np.float32)
    u = rng.random(M).astype(np.float32)
    u[:3] = [0.0, np.float32(1.0 - 2 ** -24), 0.5]
    check_against_oracle(lg, temp, k, p, u, f"V={V}")


def test_sampler_with_many_equal_logits():
    """Logits that take a dozen distinct values: the k-th largest is tied hundreds or thousands of times (every tie
    is kept), the candidate list overflows for the wide ties, and temperatures above 1 merge neighbouring values."""
    print("sampler: heavy ties", flush=True)
    V, M = 20000, 32
    g = torch.Generator().manual_seed(77)
    lg = torch.round(torch.randn(M, V, generator=g) * 1.5).to(torch.float32)
    lg[:8] += (torch.randn(8, V, generator=g) * 1e-6).to(torch.float32)       # nearly equal instead of equal
    rng = np.random.default_rng(77)
    temp = rng.choice([0.7, 1.0, 1.3, 3.0], size=M).astype(np.float32)
    k = rng.choice([1, 5, 50, 500, 3000], size=M).astype(np.int32)
    p = rng.choice([1.0, 0.9, 0.3], size=M).astype(np.float32)
    u = rng.random(M).astype(np.float32)
    check_against_oracle(lg, temp, k, p, u, "ties")
