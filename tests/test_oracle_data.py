"""Pins for the oracle's overlap partition and minibatch draws (CPU only).

The partition is checked against the set identities Section V-A states (D_j = O u S_j, the S_j disjoint,
|S_j| = floor((n-o)/k), their union D - O), at the paper's own sizes (n = 60000, k in {4, 8}, the overlap
ratios of its figure), and for being a uniform shuffle; the draws against exact rational arithmetic, closed
forms for special |D_j|, the already pinned Rademacher stream, and uniformity.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import dw_data as D
from oracle import dw_oracle as O


@pytest.mark.parametrize("k", [4, 8])
@pytest.mark.parametrize("ratio", [0.0, 0.125, 0.25, 0.375, 0.5])
def test_partition_identities_at_the_paper_sizes(k, ratio):
    n = 60000
    o = int(ratio * n)
    Oset, S = D.overlap_partition(n, o, k, seed=7)
    s = (n - o) // k
    assert Oset.shape == (o,) and S.shape == (k, s)
    assert len(set(Oset.tolist())) == o
    own = [set(S[j].tolist()) for j in range(k)]
    assert all(len(x) == s for x in own)
    union = set().union(*own)
    assert len(union) == k * s                                  # pairwise disjoint
    assert not (union & set(Oset.tolist()))
    # the union of the S_j is D - O, up to the (n - o) mod k points the floor leaves over
    rest = set(range(n)) - set(Oset.tolist()) - union
    assert len(rest) == (n - o) % k
    Dj = D.worker_datasets(n, o, k, seed=7)
    for j in range(k):
        assert set(Dj[j].tolist()) == set(Oset.tolist()) | own[j]


def test_partition_remainder_points_go_to_no_worker():
    n, o, k = 103, 10, 4                                        # 93 = 4*23 + 1
    Oset, S = D.overlap_partition(n, o, k, seed=3)
    assert S.shape == (4, 23)
    used = set(Oset.tolist()) | set(S.reshape(-1).tolist())
    assert len(used) == 10 + 92 and used < set(range(n))


def test_partition_degenerate_sizes():
    Oset, S = D.overlap_partition(16, 16, 4, seed=1)            # everything shared
    assert sorted(Oset.tolist()) == list(range(16)) and S.shape == (4, 0)
    Oset, S = D.overlap_partition(16, 0, 1, seed=1)             # one worker owns it all
    assert Oset.size == 0 and sorted(S[0].tolist()) == list(range(16))
    Oset, S = D.overlap_partition(3, 0, 8, seed=1)              # fewer points than workers
    assert S.shape == (8, 0)


def test_partition_follows_the_key_order_and_the_seed():
    n = 500
    keys = D.partition_keys(n, seed=11)
    assert len(set(keys)) == n
    Oset, S = D.overlap_partition(n, 100, 4, seed=11)
    order = np.concatenate([Oset, S.reshape(-1)])
    kk = [keys[i] for i in order]
    assert kk == sorted(kk)                                     # ascending keys, by an independent check
    assert kk[0] == min(keys) and kk[-1] == max(keys)
    other, _ = D.overlap_partition(n, 100, 4, seed=12)
    assert other.tolist() != Oset.tolist()
    # the keys are the SplitMix64 sequence started from mix(seed)
    np.testing.assert_array_equal(np.array(keys[:20], dtype=np.uint64), O.splitmix_stream(O._mix64(11), 20))


def test_partition_ties_are_broken_by_index(monkeypatch):
    monkeypatch.setattr(D, "partition_keys", lambda n, seed: [5, 1, 5, 1, 0, 5])
    Oset, S = D.overlap_partition(6, 2, 2, seed=0)
    assert Oset.tolist() == [4, 1] and S.tolist() == [[3, 0], [2, 5]]


def test_partition_is_a_uniform_shuffle():
    # membership of a fixed point in O over many seeds: binomial with p = o/n
    n, o, trials = 40, 10, 2000
    hits = sum(0 in D.overlap_partition(n, o, 3, seed=s)[0].tolist() for s in range(trials))
    p = o / n
    assert abs(hits - trials * p) < 5 * np.sqrt(trials * p * (1 - p))
    # position of point 0 in the permutation (o = n): chi-square over n cells
    n, trials = 10, 4000
    cnt = np.zeros(n)
    for s in range(trials):
        cnt[D.overlap_partition(n, n, 1, seed=1000 + s)[0].tolist().index(0)] += 1
    chi2 = ((cnt - trials / n) ** 2 / (trials / n)).sum()
    assert chi2 < 33.7                                          # 9 degrees of freedom, p = 1e-4


def test_batch_positions_are_the_exact_scaled_draws():
    seed, j, t, B, m = 99, 2, 5, 64, 52500
    pos = D.batch_positions(seed, j, t, B, m)
    words = O.rademacher_words(seed, j, t, 64 * B)              # the pinned stream: word b is draw b
    for b in range(B):
        u = int(words[b])
        assert pos[b] == int(Fraction(u, 2 ** 64) * m // 1)
    assert pos.min() >= 0 and pos.max() < m


def test_batch_positions_special_sizes():
    seed, j, t, B = 4, 1, 0, 256
    assert not D.batch_positions(seed, j, t, B, 1).any()        # a single point: always that point
    words = O.rademacher_words(seed, j, t, 64 * B)
    top3 = (words >> np.uint64(61)).astype(np.int64)
    np.testing.assert_array_equal(D.batch_positions(seed, j, t, B, 8), top3)     # |D_j| = 2^3: the top 3 bits
    # |D_j| = 2: the top bit, which is the sign of element 64b+63 of the Rademacher vector of the same key
    z = O.words_to_signs(words, 64 * B)
    np.testing.assert_array_equal(D.batch_positions(seed, j, t, B, 2), (z[63::64] > 0).astype(np.int64))


def test_batch_positions_are_uniform_and_differ_between_workers_and_steps():
    m, B = 12, 6000
    pos = D.batch_positions(5, 0, 0, B, m)
    cnt = np.bincount(pos, minlength=m)
    chi2 = ((cnt - B / m) ** 2 / (B / m)).sum()
    assert chi2 < 39.0                                          # 11 degrees of freedom, p = 1e-4
    a = D.batch_positions(5, 0, 0, 64, 10 ** 6)
    assert (a != D.batch_positions(5, 1, 0, 64, 10 ** 6)).mean() > 0.9
    assert (a != D.batch_positions(5, 0, 1, 64, 10 ** 6)).mean() > 0.9
    assert (a != D.batch_positions(6, 0, 0, 64, 10 ** 6)).mean() > 0.9


def test_draw_batch_gathers_rows_and_labels_of_the_workers_own_points():
    n, o, k, B = 200, 40, 4, 32
    rng = np.random.default_rng(0)
    data = rng.standard_normal((n, 5))
    labels = rng.integers(0, 10, size=n)
    Dj = D.worker_datasets(n, o, k, seed=21)
    steps = [0, 3, 3, 7]
    x, y = D.draw_batch(data, labels, Dj, seed=77, steps=steps, batch=B)
    assert x.shape == (k, B, 5) and y.shape == (k, B)
    for j in range(k):
        own = set(Dj[j].tolist())
        for b in range(B):
            hit = [i for i in own if np.array_equal(data[i], x[j, b])]
            assert len(hit) == 1 and labels[hit[0]] == y[j, b]
    # equal local steps do not mean equal draws: workers 1 and 2 have streams of their own
    p1 = D.batch_positions(77, 1, 3, B, Dj.shape[1])
    p2 = D.batch_positions(77, 2, 3, B, Dj.shape[1])
    assert (p1 != p2).any()
