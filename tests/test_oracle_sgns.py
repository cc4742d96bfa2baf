"""Pins for the oracle's SGNS step and loss (Algorithm 1, embedding-training loop).

The update is SGD ascent on J = sum_b [log s(x.c0) + sum_k log s(-x.ck)] evaluated at the pre-batch
tables and summed over the batch, so (table' - table) / lr must equal the gradient of J: checked by
central finite differences and by torch-CPU autograd (both independent of the oracle's code).  The loss
has closed forms for hand-made tables, and the first batch from a zero context table has one too.
"""
import math

import numpy as np
import pytest
import torch

import oracle


def J_fp64(X, C, pairs, neg):
    X = np.asarray(X, dtype=np.float64); C = np.asarray(C, dtype=np.float64)
    tot = 0.0
    for b in range(pairs.shape[0]):
        x = X[pairs[b, 0]]
        tot += -math.log1p(math.exp(-float(x @ C[pairs[b, 1]])))
        for k in range(neg.shape[1]):
            tot += -math.log1p(math.exp(float(x @ C[neg[b, k]])))
    return tot


def tiny_case(seed=0, V=8, d=4, B=6, K=2):
    rng = np.random.default_rng(seed)
    X = rng.normal(0, 0.7, (V, d)).astype(np.float32)
    C = rng.normal(0, 0.7, (V, d)).astype(np.float32)
    pairs = rng.integers(0, V, (B, 2)).astype(np.int32)
    pairs[1] = pairs[0]                  # duplicated pair
    pairs[2, 0] = pairs[0, 0]            # repeated src with another ctx
    neg = rng.integers(0, V, (B, K)).astype(np.int32)
    neg[0, 0] = pairs[0, 1]              # negative equal to its own positive context
    neg[3, 1] = neg[3, 0]                # the same negative twice
    neg[4, 0] = pairs[4, 0]              # negative id equal to the source id
    return X, C, pairs, neg


def test_update_equals_finite_difference_gradient():
    X, C, pairs, neg = tiny_case()
    lr = 2.0 ** -20          # small enough that fp32 storage of table+delta is the only rounding
    X1, C1 = X.copy(), C.copy()
    oracle.train_batch(X1, C1, pairs, neg, lr)
    h = 1e-6
    for T, T1, name in ((X, X1, "X"), (C, C1, "C")):
        grad = np.zeros(T.shape)
        for idx in np.ndindex(T.shape):
            Tp = T.astype(np.float64).copy(); Tm = Tp.copy()
            Tp[idx] += h; Tm[idx] -= h
            if name == "X":
                grad[idx] = (J_fp64(Tp, C, pairs, neg) - J_fp64(Tm, C, pairs, neg)) / (2 * h)
            else:
                grad[idx] = (J_fp64(X, Tp, pairs, neg) - J_fp64(X, Tm, pairs, neg)) / (2 * h)
        want = (T.astype(np.float64) + lr * grad).astype(np.float32)
        # identical up to one fp32 rounding of the final store
        assert np.abs(T1.astype(np.float64) - want.astype(np.float64)).max() <= 1.2e-7 * np.abs(want).max()
        # and the recovered gradient agrees to 1e-6 relative where the delta is resolvable
        touched = grad != 0
        assert touched.any()
        untouched_rows = ~touched.any(axis=1)
        assert np.array_equal(T1[untouched_rows], T[untouched_rows])


def test_gradient_to_1e6_with_large_lr_in_wide_tables():
    """Same check with lr = 1 on tables whose entries are exact in fp32 after the update is removed:
    compare the oracle's delta (recovered from fp32 tables scaled so rounding is < 1e-7) with FD."""
    X, C, pairs, neg = tiny_case(seed=3, V=6, d=3, B=5, K=2)
    lr = 1.0
    X1, C1 = X.copy(), C.copy()
    oracle.train_batch(X1, C1, pairs, neg, lr)
    h = 1e-6
    for T, T1, which in ((X, X1, 0), (C, C1, 1)):
        for idx in np.ndindex(T.shape):
            Tp = T.astype(np.float64).copy(); Tm = Tp.copy()
            Tp[idx] += h; Tm[idx] -= h
            args_p = (Tp, C) if which == 0 else (X, Tp)
            args_m = (Tm, C) if which == 0 else (X, Tm)
            g = (J_fp64(*args_p, pairs, neg) - J_fp64(*args_m, pairs, neg)) / (2 * h)
            got = float(T1[idx]) - float(T[idx])
            assert abs(got - lr * g) <= 1e-6 * max(1.0, abs(g)) + 1.5e-7 * abs(float(T1[idx]))


def test_update_equals_torch_autograd():
    rng = np.random.default_rng(5)
    V, d, B, K = 50, 16, 200, 5
    X = rng.normal(0, 0.3, (V, d)).astype(np.float32)
    C = rng.normal(0, 0.3, (V, d)).astype(np.float32)
    pairs = rng.integers(0, V, (B, 2)).astype(np.int32)
    neg = rng.integers(0, V, (B, K)).astype(np.int32)
    lr = 0.05
    Xt = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    Ct = torch.tensor(C, dtype=torch.float64, requires_grad=True)
    src = torch.tensor(pairs[:, 0], dtype=torch.long)
    ctx = torch.tensor(pairs[:, 1], dtype=torch.long)
    ng = torch.tensor(neg, dtype=torch.long)
    x = Xt[src]
    s0 = (x * Ct[ctx]).sum(-1)
    sk = (x[:, None, :] * Ct[ng]).sum(-1)
    J = torch.nn.functional.logsigmoid(s0).sum() + torch.nn.functional.logsigmoid(-sk).sum()
    J.backward()
    lr32 = float(np.float32(lr))
    wantX = (Xt.detach() + lr32 * Xt.grad).numpy().astype(np.float32)
    wantC = (Ct.detach() + lr32 * Ct.grad).numpy().astype(np.float32)
    X1, C1 = X.copy(), C.copy()
    oracle.train_batch(X1, C1, pairs, neg, lr)
    # fp64 on both sides; the only difference is summation order before one fp32 rounding
    assert np.abs(X1.astype(np.float64) - wantX).max() <= 1.2e-7 * np.abs(wantX).max()
    assert np.abs(C1.astype(np.float64) - wantC).max() <= 1.2e-7 * np.abs(wantC).max()
    assert (X1 == wantX).mean() > 0.999 and (C1 == wantC).mean() > 0.999
    # loss: -J
    assert abs(oracle.eval_loss(X, C, pairs, neg) + J.item()) <= 1e-10 * abs(J.item())


def test_loss_closed_forms():
    V, d, K = 10, 8, 5
    rng = np.random.default_rng(2)
    X = rng.normal(size=(V, d)).astype(np.float32)
    C = np.zeros((V, d), dtype=np.float32)
    pairs = rng.integers(0, V, (7, 2)).astype(np.int32)
    neg = rng.integers(0, V, (7, K)).astype(np.int32)
    # all scores zero: (K+1) ln 2 per pair
    assert abs(oracle.eval_loss(X, C, pairs, neg) / 7 - (K + 1) * math.log(2)) < 1e-14
    assert abs((K + 1) * math.log(2) - 4.1588830833596715) < 1e-15
    # one-hot rows: x = a e1, c = b e1  =>  s = a b
    X[:] = 0; C[:] = 0
    X[3, 0] = 1.5; C[4, 0] = -2.0; C[5, 0] = 0.5
    pairs = np.array([[3, 4]], dtype=np.int32)
    neg = np.array([[5, 5, 4]], dtype=np.int32)
    want = math.log1p(math.exp(3.0)) + 2 * math.log1p(math.exp(0.75)) + math.log1p(math.exp(-3.0))
    assert abs(oracle.eval_loss(X, C, pairs, neg) - want) < 1e-13
    # large |s| stays finite (stable softplus)
    X[3, 0] = 300.0
    assert math.isfinite(oracle.eval_loss(X, C, pairs, neg))


def test_first_batch_from_zero_context_closed_form():
    """C = 0: every score is 0, g0 = 1/2, gk = -1/2, so X is unchanged bit for bit and
    C'[r] = (lr/2) (sum of x_src over pairs with ctx = r  -  sum of x_src over negatives = r)."""
    V, d, B, K = 300, 32, 1000, 5
    X, C = oracle.init_tables(V, d, seed=0)
    rng = np.random.default_rng(9)
    pairs = rng.integers(0, V, (B, 2)).astype(np.int32)
    neg = rng.integers(0, V // 3, (B, K)).astype(np.int32)
    lr = 0.025
    X1, C1 = X.copy(), C.copy()
    oracle.train_batch(X1, C1, pairs, neg, lr)
    assert np.array_equal(X1, X)
    want = np.zeros((V, d))
    half = float(np.float32(lr)) / 2
    np.add.at(want, pairs[:, 1], half * X[pairs[:, 0]].astype(np.float64))
    for k in range(K):
        np.add.at(want, neg[:, k], -half * X[pairs[:, 0]].astype(np.float64))
    assert np.abs(C1 - want.astype(np.float32)).max() <= 1e-7 * np.abs(want).max()
    untouched = np.setdiff1d(np.arange(V), np.concatenate([pairs[:, 1], neg.reshape(-1)]))
    assert untouched.size > 0 and not C1[untouched].any()


def test_minibatch_synchronous_semantics():
    rng = np.random.default_rng(4)
    V, d, B, K = 20, 8, 64, 3
    X = rng.normal(0, 0.5, (V, d)).astype(np.float32)
    C = rng.normal(0, 0.5, (V, d)).astype(np.float32)
    pairs = rng.integers(0, V, (B, 2)).astype(np.int32)
    neg = rng.integers(0, V, (B, K)).astype(np.int32)
    lr = 0.1
    Xa, Ca = X.copy(), C.copy()
    oracle.train_batch(Xa, Ca, pairs, neg, lr)
    # permuting the pairs together with their negatives changes nothing beyond fp64 rounding
    perm = rng.permutation(B)
    Xb, Cb = X.copy(), C.copy()
    oracle.train_batch(Xb, Cb, pairs[perm].copy(), neg[perm].copy(), lr)
    assert np.abs(Xa - Xb).max() <= 1.2e-7 * np.abs(Xa).max()
    assert np.abs(Ca - Cb).max() <= 1.2e-7 * np.abs(Ca).max()
    # two half batches in sequence are a different (second-order different) computation
    Xc, Cc = X.copy(), C.copy()
    oracle.train_batch(Xc, Cc, pairs[:B // 2].copy(), neg[:B // 2].copy(), lr)
    oracle.train_batch(Xc, Cc, pairs[B // 2:].copy(), neg[B // 2:].copy(), lr)
    diff = np.abs(Xa - Xc).max()
    assert 1e-5 < diff < 0.5
    # empty batch is a no-op
    Xd, Cd = X.copy(), C.copy()
    oracle.train_batch(Xd, Cd, np.zeros((0, 2), np.int32), np.zeros((0, K), np.int32), lr)
    assert np.array_equal(Xd, X) and np.array_equal(Cd, C)


def test_init_tables():
    V, d = 2000, 128
    X, C = oracle.init_tables(V, d, seed=0)
    assert not C.any()
    assert X.min() > -0.5 / d and X.max() < 0.5 / d
    assert abs(X.mean()) < 4 * (1 / d) / math.sqrt(12 * V * d)
    assert abs(X.var() - (1 / d) ** 2 / 12) < 0.01 * (1 / d) ** 2 / 12
    # every value is (m + 0.5) 2^-23 - 0.5 over d for a 23-bit m: recover m exactly
    m = (X.astype(np.float64) * d + 0.5) * 2**23 - 0.5
    assert np.abs(m - np.round(m)).max() < 1e-6 and m.min() >= 0 and m.max() <= 2**23 - 1
    # m is the top 23 bits of the Philox word for (row, col//4), stream 1, word col%4
    for row, col in ((0, 0), (5, 3), (1999, 127), (77, 64)):
        r = oracle.philox4x32_10([row, 0, col // 4, 1], [0, 0])[col % 4]
        assert int(round(m[row, col])) == int(r) >> 9
    # different seed, different table; d not a power of two still inside the interval
    X2, _ = oracle.init_tables(50, 100, seed=1)
    assert X2.min() > -0.5 / 100 and X2.max() < 0.5 / 100
    assert not np.array_equal(X2[:, :100], oracle.init_tables(50, 100, seed=2)[0])


@pytest.mark.parametrize("threads", [1, 2, 3, 8, 100])
def test_threaded_step_equals_the_plain_step(threads):
    """oracle_train_batch_threads (used only to time the oracle on all cores) against the pinned plain step:
    the same fp64 terms, summed per thread and then across threads, so the fp32 results agree to the last
    bit except where a sum lands within 1e-16 of a rounding boundary."""
    rng = np.random.default_rng(threads)
    V, d, B, K = 300, 12, 257, 4
    X = rng.normal(0, 0.4, (V, d)).astype(np.float32)
    C = rng.normal(0, 0.4, (V, d)).astype(np.float32)
    pairs = np.minimum((rng.pareto(0.8, (B, 2)) * 10).astype(np.int64), V - 1).astype(np.int32)   # hubs: rows repeat
    neg = rng.integers(0, V, (B, K)).astype(np.int32)
    X1, C1, X2, C2 = X.copy(), C.copy(), X.copy(), C.copy()
    oracle.train_batch(X1, C1, pairs, neg, 0.05)
    oracle.train_batch_threads(X2, C2, pairs, neg, 0.05, threads)
    assert not np.array_equal(X1, X)
    for a, b in ((X1, X2), (C1, C2)):
        assert np.abs(a.astype(np.float64) - b).max() <= 1.2e-7 * np.abs(a).max()
        assert (a.view(np.uint32) != b.view(np.uint32)).mean() < 1e-3
    untouched = np.ones(V, bool); untouched[pairs[:, 1]] = False; untouched[neg.reshape(-1)] = False
    assert np.array_equal(C2[untouched].view(np.uint32), C[untouched].view(np.uint32))
    with pytest.raises(ValueError):
        oracle.train_batch_threads(X2, C2, np.array([[0, V]], np.int32), neg[:1], 0.05, 2)
