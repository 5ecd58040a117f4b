"""Pins of the first/last-stage oracle (oracle/head_oracle.py): values fixed by the definitions themselves
(section 2.1 of the paper: embedding, projection to logits, greedy / top-k / nucleus sampling), special cases in
which the sampler must reduce to something simpler, and brute force on small vocabularies."""
import numpy as np
import pytest

from oracle import head_oracle as Hd


def bits(x):
    x = np.asarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def test_embedding_copies_rows_and_zeroes_unknown_ids():
    table = bits(np.arange(12, dtype=np.float32).reshape(4, 3))
    out = Hd.embedding(table, np.array([2, 0, 3, 7, -1]))
    assert np.array_equal(out[:3], table[[2, 0, 3]]) and not out[3:].any()


def test_final_logits_closed_forms():
    H, V = 8, 5
    x = np.zeros((3, H)); x[0] = 2.0; x[1] = np.arange(1, H + 1); x[2] = -3.0
    gamma = bits(np.full(H, 1.0)); w = bits(np.eye(V, H))
    lg = Hd.final_logits(x, [0, 1, 2], gamma, w, 0.0)
    # a constant row normalises to +-1 whatever its scale; the identity projection then returns the normalised entries
    assert np.allclose(lg[0], 1.0) and np.allclose(lg[2], -1.0)
    r = np.arange(1, H + 1) / np.sqrt(np.mean(np.arange(1, H + 1) ** 2.0))
    assert np.allclose(lg[1], r[:V])
    # gains multiply after normalisation; rows are selected by index; eps sits inside the root
    gamma2 = bits(np.array([2.0, 1, 1, 1, 1, 1, 1, 1]))
    assert np.isclose(Hd.final_logits(x, [1], gamma2, w, 0.0)[0, 0], 2 * r[0])
    assert np.allclose(Hd.final_logits(x, [2, 0], gamma, w, 0.0), lg[[2, 0]])
    assert np.allclose(Hd.final_logits(x, [0], gamma, w, 12.0)[0], 2.0 / np.sqrt(4.0 + 12.0))


def test_greedy_takes_the_first_maximum():
    assert Hd.greedy(np.array([0.1, 3.0, -1.0, 3.0])) == 1
    assert Hd.sample(np.array([0.1, 3.0, -1.0, 3.0]), 0.0, 0, 1.0, 0.99) == 1


def test_sampler_reduces_to_greedy():
    rng = np.random.default_rng(0)
    lg = rng.normal(size=50)
    for u in (0.0, 0.3, 0.999):
        assert Hd.sample(lg, 1.0, 1, 1.0, u) == Hd.greedy(lg)             # top-1
        assert Hd.sample(lg, 1.0, 0, 1e-9, u) == Hd.greedy(lg)            # a vanishing nucleus
        assert Hd.sample(lg, 1e-4, 0, 1.0, u) == Hd.greedy(lg)            # a vanishing temperature


def test_full_distribution_is_the_inverse_cdf_of_softmax():
    """top_k = V, top_p = 1, temperature 1: sweeping u over a fine grid must hit every token with a frequency equal
    to its softmax probability, in index order."""
    lg = np.array([0.0, 1.0, -2.0, 0.5, 3.0])
    p = np.exp(lg) / np.exp(lg).sum()
    n = 20000
    picks = np.array([Hd.sample(lg, 1.0, 0, 1.0, (i + 0.5) / n) for i in range(n)])
    assert np.all(np.diff(picks) >= 0)                                    # index order
    assert np.allclose(np.bincount(picks, minlength=5) / n, p, atol=2.0 / n)
    shifted = np.array([Hd.sample(lg + 7.5, 1.0, 0, 1.0, (i + 0.5) / n) for i in range(0, n, 97)])
    assert np.array_equal(shifted, picks[::97])                           # softmax ignores a common shift
    hot = np.array([Hd.sample(lg, 0.5, 0, 1.0, (i + 0.5) / n) for i in range(n)])
    p2 = np.exp(2 * lg) / np.exp(2 * lg).sum()
    assert np.allclose(np.bincount(hot, minlength=5) / n, p2, atol=2.0 / n)   # temperature divides the logits


def test_top_k_and_nucleus_sets():
    lg = np.log(np.array([0.05, 0.4, 0.1, 0.25, 0.2]))
    keep, p = Hd.kept_distribution(lg, 1.0, 2, 1.0)
    assert keep.tolist() == [False, True, False, True, False] and np.allclose(p[[1, 3]], [0.4 / 0.65, 0.25 / 0.65])
    keep, p = Hd.kept_distribution(lg, 1.0, 0, 0.6)                        # 0.4 + 0.25 = 0.65 >= 0.6 first
    assert keep.tolist() == [False, True, False, True, False]
    keep, p = Hd.kept_distribution(lg, 1.0, 0, 0.65 + 1e-9)                # now the third token is needed
    assert keep.tolist() == [False, True, False, True, True] and np.isclose(p.sum(), 1.0)
    keep, _ = Hd.kept_distribution(lg, 1.0, 3, 0.5)                        # top-k first, then the nucleus inside it
    assert keep.tolist() == [False, True, False, True, False]             # 0.4/0.85 < 0.5 <= (0.4+0.25)/0.85
    # ties are kept whole
    tie = np.log(np.array([0.3, 0.3, 0.2, 0.2]))
    assert Hd.kept_distribution(tie, 1.0, 1, 1.0)[0].tolist() == [True, True, False, False]
    assert Hd.kept_distribution(tie, 1.0, 0, 0.7)[0].tolist() == [True, True, True, True]


@pytest.mark.parametrize("seed", range(5))
def test_nucleus_is_minimal_and_sufficient_on_random_logits(seed):
    rng = np.random.default_rng(seed)
    lg = rng.normal(scale=2.0, size=200)
    base = np.exp(lg - lg.max()); base /= base.sum()
    for top_p in (0.1, 0.5, 0.9, 0.99):
        keep, p = Hd.kept_distribution(lg, 1.0, 0, top_p)
        mass = base[keep].sum()
        assert mass >= top_p - 1e-12
        assert mass - base[keep].min() < top_p                             # dropping the least probable kept token falls short
        assert base[~keep].max(initial=0.0) <= base[keep].min()            # only the most probable tokens are kept
        for u in rng.random(20):
            assert keep[Hd.sample(lg, 1.0, 0, top_p, float(u))]
