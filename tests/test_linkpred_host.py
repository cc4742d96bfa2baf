"""Host-side bookkeeping of the link-prediction harness (Sec. V-B): edge-list reading, the split, non-edge
sampling and the AUC, each against a definition written out by brute force."""
import itertools

import numpy as np

from paper_2005_13789_amd import linkpred as lp


def test_auc_equals_pair_counting_with_ties():
    rng = np.random.default_rng(0)
    for _ in range(20):
        pos = rng.integers(0, 6, rng.integers(1, 30)).astype(np.float64)
        neg = rng.integers(0, 6, rng.integers(1, 30)).astype(np.float64)
        wins = sum(1.0 if p > n else 0.5 if p == n else 0.0 for p, n in itertools.product(pos, neg))
        assert abs(lp.auc(pos, neg) - wins / (pos.size * neg.size)) < 1e-12
    assert lp.auc([3.0, 2.0], [1.0, 0.0]) == 1.0 and lp.auc([0.0], [1.0, 2.0]) == 0.0 and lp.auc([1.0], [1.0]) == 0.5


def test_read_edge_list_renumbers_in_order_of_first_appearance(tmp_path):
    f = tmp_path / "edges.txt"
    f.write_text("# comment\n10 20\n20 7\n% other comment\n7 10 0.5\n99 10\n")
    edges, n = lp.read_edge_list(str(f))
    assert n == 4
    assert edges.tolist() == [[0, 1], [1, 2], [2, 0], [3, 0]]


def test_split_is_a_partition_of_the_distinct_undirected_edges():
    edges = np.array([[1, 2], [2, 1], [3, 3], [0, 4], [4, 5], [5, 6], [1, 2], [6, 0], [2, 3], [7, 1], [8, 2]])
    train, test = lp.split_edges(edges, 0.25, seed=1)
    both = np.concatenate([train, test])
    want = {(1, 2), (0, 4), (4, 5), (5, 6), (0, 6), (2, 3), (1, 7), (2, 8)}
    assert {tuple(e) for e in both.tolist()} == want and both.shape[0] == len(want)
    assert test.shape[0] == 2
    t2, s2 = lp.split_edges(edges, 0.25, seed=1)
    assert np.array_equal(train, t2) and np.array_equal(test, s2)


def test_non_edges_are_not_edges():
    rng = np.random.default_rng(2)
    V = 30
    edges = rng.integers(0, V, (300, 2))                 # dense: most random pairs are edges
    pairs = lp.sample_non_edges(V, edges, 50, seed=3)
    have = {(min(a, b), max(a, b)) for a, b in edges.tolist()}
    assert pairs.shape == (50, 2)
    for a, b in pairs.tolist():
        assert a != b and (min(a, b), max(a, b)) not in have
