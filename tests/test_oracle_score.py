"""Pins of the oracle's pair score (evaluation for link prediction, Sec. V-B): hand values, the choice of
the second table, and agreement with the loss function, whose single positive term is softplus(-score)."""
import numpy as np

import oracle


def test_score_hand_values_and_table_choice():
    X = np.array([[1, 2, 3, 4], [0.5, 0, 0, 0], [0, 0, 1, 0]], np.float32)
    C = np.array([[4, 3, 2, 1], [0, 7, 0, 0], [1, 1, 1, 1]], np.float32)
    pairs = np.array([[0, 0], [0, 1], [1, 2], [2, 0], [0, 2]], np.int32)
    # vertex . context:  1*4+2*3+3*2+4*1 = 20 ;  2*7 = 14 ;  0.5 ;  2 ;  10
    assert np.array_equal(oracle.score_pairs(X, C, pairs, True), [20.0, 14.0, 0.5, 2.0, 10.0])
    # vertex . vertex:   1+4+9+16 = 30 ;  0.5 ;  0 ;  3 ;  3
    assert np.array_equal(oracle.score_pairs(X, C, pairs, False), [30.0, 0.5, 0.0, 3.0, 3.0])
    assert oracle.score_pairs(X, C, pairs[:0], True).shape == (0,)


def test_score_agrees_with_the_positive_loss_term():
    rng = np.random.default_rng(0)
    V, d, n = 50, 24, 200
    X = rng.normal(0, 0.4, (V, d)).astype(np.float32)
    C = rng.normal(0, 0.4, (V, d)).astype(np.float32)
    pairs = rng.integers(0, V, (n, 2)).astype(np.int32)
    s = oracle.score_pairs(X, C, pairs, True)
    none = np.empty((1, 0), np.int32)
    for i in range(n):
        loss = oracle.eval_loss(X, C, pairs[i:i + 1], none)          # K = 0: softplus(-s)
        assert abs(-np.log(np.expm1(loss)) - s[i]) <= 1e-9 * max(1.0, abs(s[i]))
