"""Pins for the oracle's other down-sampling rules (Sec. 3.2: random, percentile, max-reward) and
for the "Before" advantage normalisation (App. "On Advantage Normalization").  CPU only.

Each pin is something other than the oracle's own formula: brute force over all subsets, a
library quantile routine in the cases where every convention agrees with the reading taken, a
separation property that characterises the answer, a library z-score."""
import itertools

import numpy as np
import pytest
import scipy.stats

from oracle import pods_oracle as po
from paper_2504_13818_amd import inputs


def _groups(seed, count, n, kinds=("binary", "ternary", "cont")):
    rng = np.random.default_rng(seed)
    for i in range(count):
        kind = kinds[i % len(kinds)]
        if kind == "binary":
            yield (rng.random(n) < rng.random()).astype(np.float32)
        elif kind == "ternary":
            yield rng.integers(0, 3, n).astype(np.float32) / 2
        else:
            yield rng.normal(size=n).astype(np.float32)


# ---- max-reward ---------------------------------------------------------------------------

def test_maxr_is_the_subset_with_the_largest_reward_sum():
    for r in _groups(1, 30, 9):
        for m in (1, 3, 8, 9):
            sel = po.downsample_maxr(r, m)
            assert len(set(sel)) == m
            best = max(sum(float(r[i]) for i in S) for S in itertools.combinations(range(len(r)), m))
            assert sum(float(r[i]) for i in sel) == best


def test_maxr_order_and_tie_rule():
    r = np.array([1, 0, 1, 1, 0, 1], dtype=np.float32)
    assert po.downsample_maxr(r, 2) == [3, 5]            # equal rewards at the cut: highest indices stay
    assert po.downsample_maxr(r, 5) == [4, 0, 2, 3, 5]   # ascending (reward, index)
    r = np.array([0.0, -0.0, 0.0], dtype=np.float32)
    assert po.downsample_maxr(r, 2) == [1, 2]            # -0.0 == +0.0


def test_maxr_is_the_top_part_of_max_variance_with_k_equal_m():
    # the k = m candidate of Alg. 2 is exactly the max-reward subset
    for r in _groups(2, 20, 12):
        ind = po.stable_argsort(r)
        assert po.downsample_maxr(r, 5) == ind[-5:]
        assert sorted(po.downsample_maxr(r, 12)) == list(range(12))


# ---- percentile ---------------------------------------------------------------------------

@pytest.mark.parametrize("n,m", [(9, 3), (15, 4), (63, 16), (255, 64), (7, 7)])
def test_perc_matches_library_quantiles_when_conventions_agree(n, m):
    # For odd n, q n = (2j-1) n / (2m) is never an integer, and then floor(q n) is also the
    # position of numpy's inverted-CDF quantile (the smallest x with F(x) >= q).
    rng = np.random.default_rng(n * 100 + m)
    r = rng.permutation(n).astype(np.float32)             # distinct values
    sel = po.downsample_perc(r, m)
    q = (np.arange(1, m + 1) - 0.5) / m
    want = np.quantile(r.astype(np.float64), q, method="inverted_cdf")
    assert np.array_equal(r[sel].astype(np.float64), want)


def test_perc_even_spacing_and_edges():
    r = np.arange(8, dtype=np.float32)
    assert po.downsample_perc(r, 2) == [2, 6]             # quantiles 1/4 and 3/4 of 0..7
    assert po.downsample_perc(r, 8) == list(range(8))     # m = n keeps everything
    assert po.downsample_perc(r, 1) == [4]                # the median position
    r = np.arange(256, dtype=np.float32)[::-1].copy()     # descending input: positions map through the sort
    sel = po.downsample_perc(r, 64)
    assert [int(r[i]) for i in sel] == [4 * j + 2 for j in range(64)]


def test_perc_positions_distinct_and_increasing():
    for n, m in [(5, 5), (6, 5), (64, 16), (100, 33), (256, 64), (257, 256)]:
        r = np.arange(n, dtype=np.float32)
        sel = po.downsample_perc(r, m)
        assert all(a < b for a, b in zip(sel, sel[1:]))
        # pick j is one of the elements that overlap the j-th of m equal-mass bins of the sorted order
        for j, p in enumerate(sel):
            assert (j * n) // m <= p <= -((-(j + 1) * n) // m) - 1


def test_perc_ties_follow_the_index_order():
    r = np.array([1, 0, 1, 0, 1, 0], dtype=np.float32)    # sorted order: 1 3 5 0 2 4
    assert po.downsample_perc(r, 3) == [3, 0, 4]           # positions 1, 3, 5


# ---- random -------------------------------------------------------------------------------

def test_rand_separation_property():
    rng = np.random.default_rng(5)
    for _ in range(50):
        n = int(rng.integers(1, 40))
        m = int(rng.integers(1, n + 1))
        keys = rng.integers(0, 6 if rng.random() < 0.5 else 2**32, n, dtype=np.uint64).astype(np.uint32)
        sel = po.downsample_rand(keys, m)
        assert len(set(sel)) == m
        inside = [(int(keys[i]), i) for i in sel]
        outside = [(int(keys[i]), i) for i in range(n) if i not in set(sel)]
        assert inside == sorted(inside)
        if outside:
            assert max(inside) < min(outside)              # characterises "the m smallest (key, index)"


def test_rand_is_uniform_over_subsets():
    # all C(5,2) = 10 subsets equally likely under iid keys: chi-square against the uniform law
    rng = np.random.default_rng(6)
    counts = {}
    trials = 20000
    for _ in range(trials):
        keys = rng.integers(0, 2**32, 5, dtype=np.uint64).astype(np.uint32)
        S = tuple(sorted(po.downsample_rand(keys, 2)))
        counts[S] = counts.get(S, 0) + 1
    assert len(counts) == 10
    chi2 = sum((c - trials / 10) ** 2 / (trials / 10) for c in counts.values())
    assert chi2 < 33.7                                     # 99.99 % point of chi-square with 9 d.o.f.


def test_rand_ignores_rewards_and_batches():
    r = inputs.rewards(0)
    rng = np.random.default_rng(7)
    keys = rng.integers(0, 2**32, r.shape, dtype=np.uint64).astype(np.uint32)
    sel = po.downsample_batch(r, 4, "rand", keys)
    sel2 = po.downsample_batch(np.zeros_like(r), 4, "rand", keys)
    assert np.array_equal(sel, sel2)
    for rule in ("maxr", "perc"):
        out = po.downsample_batch(r, 4, rule)
        assert out.shape == (r.shape[0], 4) and out.dtype == np.int32
        assert out.min() >= 0 and out.max() < r.shape[1]


# ---- "Before" normalisation ------------------------------------------------------------------

def test_before_is_the_library_zscore_of_the_whole_group():
    rng = np.random.default_rng(8)
    r = rng.normal(size=(6, 16)).astype(np.float32)
    sel, _ = po.select_batch(r, 4)
    z = scipy.stats.zscore(r.astype(np.float64), axis=1, ddof=0)
    assert np.allclose(po.advantage_before(r, sel), np.take_along_axis(z, sel.astype(np.int64), axis=1),
                       rtol=0, atol=1e-13)


def test_before_hand_worked_and_relations():
    r = np.array([[2, 4, 4, 4, 5, 5, 7, 9]], dtype=np.float32)       # mean 5, sigma 2
    sel = np.array([[0, 7, 4]], dtype=np.int32)
    assert np.allclose(po.advantage_before(r, sel), [[-1.5, 2.0, 0.0]], rtol=0, atol=1e-15)
    # keeping everything: both normalisations coincide
    full = np.arange(8, dtype=np.int32)[None]
    assert np.allclose(po.advantage_before(r, full), po.advantage(r, full), rtol=0, atol=1e-15)
    # the kept advantages generally do NOT sum to zero (the paper's argument for "After")
    assert abs(po.advantage_before(r, sel).sum()) > 0.1
    # constant group -> zeros; eps enters the denominator
    assert np.array_equal(po.advantage_before(np.full((1, 5), 0.3, np.float32), np.array([[1, 2]], np.int32)), [[0, 0]])
    assert np.allclose(po.advantage_before(r, sel, std_eps=2.0), [[-0.75, 1.0, 0.0]])


# ---- concatenation of the kept rollouts ------------------------------------------------------

def test_gather_kept_is_fancy_indexing():
    rng = np.random.default_rng(9)
    B, n, m = 5, 7, 3
    rec = rng.integers(0, 1000, (B, n, 4)).astype(np.int32)
    sel = np.stack([rng.choice(n, m, replace=False) for _ in range(B)]).astype(np.int32)
    want = rec[np.arange(B)[:, None], sel].reshape(B * m, 4)          # library indexing
    assert np.array_equal(po.gather_kept(rec, sel), want)
    lens = rng.integers(0, 50, (B, n)).astype(np.int32)              # one scalar per rollout
    assert np.array_equal(po.gather_kept(lens, sel), np.take_along_axis(lens, sel.astype(np.int64), axis=1).reshape(-1))
