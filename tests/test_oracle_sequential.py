"""Pins for the oracle's per-sample (sequential) SGD: it must equal the pinned minibatch oracle applied
to one pair at a time, and, when no row is named twice, the minibatch oracle applied to the whole batch."""
import numpy as np

import oracle


def test_sequential_equals_batches_of_one():
    rng = np.random.default_rng(0)
    V, d, B, K = 30, 8, 200, 3
    X = rng.normal(0, 0.5, (V, d)).astype(np.float32)
    C = rng.normal(0, 0.5, (V, d)).astype(np.float32)
    pairs = rng.integers(0, V, (B, 2)).astype(np.int32)
    neg = rng.integers(0, V, (B, K)).astype(np.int32)
    Xa, Ca = X.copy(), C.copy()
    oracle.train_sequential(Xa, Ca, pairs, neg, 0.1)
    Xb, Cb = X.copy(), C.copy()
    for b in range(B):
        oracle.train_batch(Xb, Cb, pairs[b:b + 1].copy(), neg[b:b + 1].copy(), 0.1)
    # identical up to the double rounding of a row that one sample names twice
    assert np.abs(Xa - Xb).max() <= 2.4e-7 * np.abs(Xb).max()
    assert np.abs(Ca - Cb).max() <= 2.4e-7 * np.abs(Cb).max()
    # and it is not the minibatch result
    Xc, Cc = X.copy(), C.copy()
    oracle.train_batch(Xc, Cc, pairs, neg, 0.1)
    assert np.abs(Xa - Xc).max() > 1e-3


def test_sequential_equals_minibatch_without_collisions():
    rng = np.random.default_rng(1)
    V, d, B, K = 4000, 16, 100, 4
    X = rng.normal(0, 0.5, (V, d)).astype(np.float32)
    C = rng.normal(0, 0.5, (V, d)).astype(np.float32)
    perm = rng.permutation(V).astype(np.int32)
    pairs = np.stack([perm[:B], perm[B:2 * B]], axis=1).copy()           # distinct sources, distinct contexts
    neg = perm[2 * B:2 * B + B * K].reshape(B, K).copy()                  # distinct from each other and from ctx
    Xa, Ca = X.copy(), C.copy()
    oracle.train_sequential(Xa, Ca, pairs, neg, 0.05)
    Xb, Cb = X.copy(), C.copy()
    oracle.train_batch(Xb, Cb, pairs, neg, 0.05)
    assert np.array_equal(Xa, Xb) and np.array_equal(Ca, Cb)
