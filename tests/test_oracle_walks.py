"""Pins of the oracle's walk augmentation (Algorithm 1, "network augmentation"): a worked example, the sample
count of full walks, and the set of samples against a definition written out by brute force."""
import numpy as np

import oracle


def test_worked_example():
    # one walk a b c d with window 2: (a,b) (a,c) (b,c) (b,d) (c,d); sample index (i*2 + j-1)
    walks = np.array([[10, 11, 12, 13]], np.int32)
    pairs, sample = oracle.walk_pairs(walks, 2)
    assert pairs.tolist() == [[10, 11], [10, 12], [11, 12], [11, 13], [12, 13]]
    assert sample.tolist() == [0, 1, 2, 3, 4]
    # a second, shorter walk padded with -1: its samples are numbered from 1 * 4 * 2
    walks = np.array([[10, 11, 12, 13], [5, 6, -1, -1]], np.int32)
    pairs, sample = oracle.walk_pairs(walks, 2)
    assert pairs.tolist()[5:] == [[5, 6]] and sample.tolist()[5:] == [8]


def test_sample_count_of_full_walks():
    rng = np.random.default_rng(0)
    for L, w in ((80, 5), (40, 5), (80, 10), (7, 3), (3, 5)):
        walks = rng.integers(0, 1000, (11, L)).astype(np.int32)
        pairs, sample = oracle.walk_pairs(walks, w)
        per_walk = sum(max(L - j, 0) for j in range(1, w + 1))      # 385 for (80, 5): the figure of config 2
        assert pairs.shape[0] == 11 * per_walk
        assert np.all(np.diff(sample) > 0) and sample.max() < 11 * L * w
    assert sum(80 - j for j in range(1, 6)) == 385


def test_samples_against_brute_force_with_holes():
    rng = np.random.default_rng(1)
    n, L, w = 9, 13, 4
    walks = rng.integers(0, 50, (n, L)).astype(np.int32)
    walks[rng.random((n, L)) < 0.2] = -1                            # holes anywhere, not only at the end
    pairs, sample = oracle.walk_pairs(walks, w)
    want = {}
    for r in range(n):
        for i in range(L):
            for k in range(i + 1, L):
                if k - i <= w and walks[r, i] >= 0 and walks[r, k] >= 0:
                    want[(r * L + i) * w + (k - i - 1)] = (int(walks[r, i]), int(walks[r, k]))
    got = {int(s): (int(a), int(b)) for s, (a, b) in zip(sample, pairs)}
    assert got == want
    # the earlier node is the source
    for s, (a, b) in got.items():
        p, j = divmod(s, w)
        r, i = divmod(p, L)
        assert walks[r, i] == a and walks[r, i + j + 1] == b
