"""Pins for the oracle's shared-negative step.

Without bf16 rounding the update is lr times the gradient of
J = sum_b [log s(x_b.c_ctx) + neg_scale sum_n log s(-x_b.c_n)]: checked by torch-CPU fp64 autograd and
by finite differences.  With rounding, the same quantities are rebuilt here from torch's own
float32 -> bfloat16 conversion (an independent rounding routine) and fp64 matmuls.
"""
import math

import numpy as np
import torch

import oracle


def case(seed, V=40, d=16, B=24, N=10):
    rng = np.random.default_rng(seed)
    X = rng.normal(0, 0.4, (V, d)).astype(np.float32)
    C = rng.normal(0, 0.4, (V, d)).astype(np.float32)
    pairs = rng.integers(0, V, (B, 2)).astype(np.int32)
    pairs[1] = pairs[0]
    negs = rng.integers(0, V, N).astype(np.int32)
    negs[1] = negs[0]                # the same negative drawn twice
    negs[2] = pairs[0, 1]            # a negative equal to a positive context
    negs[3] = pairs[2, 0]            # a negative id equal to a source id
    return X, C, pairs, negs


def test_shared_equals_autograd_without_rounding():
    X, C, pairs, negs = case(0)
    lr, scale = 0.05, 5 / 10
    Xt = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    Ct = torch.tensor(C, dtype=torch.float64, requires_grad=True)
    x = Xt[torch.tensor(pairs[:, 0], dtype=torch.long)]
    s0 = (x * Ct[torch.tensor(pairs[:, 1], dtype=torch.long)]).sum(-1)
    S = x @ Ct[torch.tensor(negs, dtype=torch.long)].T
    ls = torch.nn.functional.logsigmoid
    J = ls(s0).sum() + float(np.float32(scale)) * ls(-S).sum()
    J.backward()
    lr32 = float(np.float32(lr))
    wantX = (Xt.detach() + lr32 * Xt.grad).numpy()
    wantC = (Ct.detach() + lr32 * Ct.grad).numpy()
    X1, C1 = X.copy(), C.copy()
    loss = oracle.train_batch_shared(X1, C1, pairs, negs, lr, scale, bf16_inputs=False)
    assert np.abs(X1 - wantX).max() <= 1.2e-7 * np.abs(wantX).max()
    assert np.abs(C1 - wantC).max() <= 1.2e-7 * np.abs(wantC).max()
    assert abs(loss + J.item()) <= 1e-12 * abs(J.item())


def test_shared_finite_differences_without_rounding():
    X, C, pairs, negs = case(1, V=7, d=3, B=5, N=4)
    lr, scale = 1.0, 0.25

    def J(Xa, Ca):
        tot = 0.0
        for b in range(pairs.shape[0]):
            x = Xa[pairs[b, 0]]
            tot += -math.log1p(math.exp(-float(x @ Ca[pairs[b, 1]])))
            for n in negs:
                tot += -scale * math.log1p(math.exp(float(x @ Ca[n])))
        return tot
    X1, C1 = X.copy(), C.copy()
    oracle.train_batch_shared(X1, C1, pairs, negs, lr, scale, bf16_inputs=False)
    h = 1e-6
    X64, C64 = X.astype(np.float64), C.astype(np.float64)
    for T, T1, which in ((X64, X1, 0), (C64, C1, 1)):
        for idx in np.ndindex(T.shape):
            Tp, Tm = T.copy(), T.copy()
            Tp[idx] += h; Tm[idx] -= h
            g = (J(Tp, C64) - J(Tm, C64)) / (2 * h) if which == 0 else (J(X64, Tp) - J(X64, Tm)) / (2 * h)
            got = float(T1[idx]) - float(T[idx])
            assert abs(got - lr * g) <= 1e-6 * max(1.0, abs(g)) + 1.5e-7 * abs(float(T1[idx]))


def test_shared_with_bf16_rounding_matches_torch_bfloat16():
    X, C, pairs, negs = case(2, V=60, d=32, B=50, N=16)
    lr, scale = 0.05, 5 / 16
    lr32, sc32 = float(np.float32(lr)), float(np.float32(scale))
    q = lambda a: torch.tensor(a).to(torch.bfloat16).to(torch.float64)      # torch's own RNE conversion
    src = torch.tensor(pairs[:, 0], dtype=torch.long)
    ctx = torch.tensor(pairs[:, 1], dtype=torch.long)
    ng = torch.tensor(negs, dtype=torch.long)
    X64, C64 = torch.tensor(X, dtype=torch.float64), torch.tensor(C, dtype=torch.float64)
    Xq, Cq = q(X)[src], q(C)[ng]
    S = Xq @ Cq.T
    G = (-sc32 * torch.sigmoid(S)).to(torch.float32).to(torch.bfloat16).to(torch.float64)
    s0 = (X64[src] * C64[ctx]).sum(-1)
    g0 = 1 - torch.sigmoid(s0)
    dX = torch.zeros_like(X64); dC = torch.zeros_like(C64)
    dX.index_add_(0, src, lr32 * (g0[:, None] * C64[ctx] + G @ Cq))
    dC.index_add_(0, ctx, lr32 * g0[:, None] * X64[src])
    dC.index_add_(0, ng, lr32 * (G.T @ Xq))
    wantX, wantC = (X64 + dX).numpy(), (C64 + dC).numpy()
    X1, C1 = X.copy(), C.copy()
    loss = oracle.train_batch_shared(X1, C1, pairs, negs, lr, scale, bf16_inputs=True)
    assert np.abs(X1 - wantX).max() <= 1.2e-7 * np.abs(wantX).max()
    assert np.abs(C1 - wantC).max() <= 1.2e-7 * np.abs(wantC).max()
    want_loss = torch.nn.functional.softplus(-s0).sum() + sc32 * torch.nn.functional.softplus(S).sum()
    assert abs(loss - want_loss.item()) <= 1e-12 * want_loss.item()
    # the rounding matters: the unrounded run differs, but only at bf16 scale
    X2, C2 = X.copy(), C.copy()
    oracle.train_batch_shared(X2, C2, pairs, negs, lr, scale, bf16_inputs=False)
    diff = np.abs(X2 - X1).max() / np.abs(X1 - X).max()
    assert 1e-5 < diff < 3e-2


def test_shared_closed_forms():
    V, d, B, N = 12, 8, 6, 5
    rng = np.random.default_rng(3)
    X = rng.normal(size=(V, d)).astype(np.float32)
    C = np.zeros((V, d), np.float32)
    pairs = rng.integers(0, V, (B, 2)).astype(np.int32)
    negs = rng.integers(0, V, N).astype(np.int32)
    X1, C1 = X.copy(), C.copy()
    loss = oracle.train_batch_shared(X1, C1, pairs, negs, 0.1, 0.5, bf16_inputs=True)
    assert abs(loss - B * (1 + 0.5 * N) * math.log(2)) < 1e-12      # all scores zero
    assert np.array_equal(X1, X)                                    # zero context: no vertex update
    # N = 0 reduces to the positive-only step of the per-pair oracle
    X2, C2 = X.copy(), (rng.normal(size=(V, d)) * 0.3).astype(np.float32)
    X3, C3 = X2.copy(), C2.copy()
    oracle.train_batch_shared(X2, C2, pairs, np.zeros(0, np.int32), 0.1, 0.5)
    oracle.train_batch(X3, C3, pairs, np.zeros((B, 0), np.int32), 0.1)
    assert np.array_equal(X2, X3) and np.array_equal(C2, C3)
    # shared negatives are counter addressed by (batch index, j), stream 2
    deg = np.arange(1, 200, dtype=np.uint32)
    thr, alias, _ = oracle.build_alias(deg)
    a = oracle.sample_shared_negatives(7, 3, 64, thr, alias, base=10)
    b = oracle.sample_shared_negatives(7, 3, 32, thr, alias, base=10)
    assert np.array_equal(a[:32], b) and a.min() >= 10 and a.max() < 209
    for j in (0, 5, 63):
        r = [int(v) for v in oracle.philox4x32_10([3, 0, j, 2], [7, 0])]
        slot = (((r[0] << 32) | r[1]) * 199) >> 64
        assert a[j] == 10 + (slot if r[2] < int(thr[slot]) else int(alias[slot]))
    assert not np.array_equal(a, oracle.sample_shared_negatives(7, 4, 64, thr, alias, base=10))
