"""GPU-vs-oracle parity of the shared-negative step (bf16 MFMA tiles) through the C ABI.

Both sides round the gathered rows and the coefficients G to bfloat16 in the same places; the GPU
accumulates the dense products in fp32 on the matrix cores, the oracle in fp64.  A last-bit difference in
a score can move one G entry by one bf16 ulp (2^-8 relative) on one side only; an entry is one of N terms
of a delta (N >= 128), i.e. at most 2^-8 / 128 = 3e-5 of it per flipped entry, so the bar is stated on the
update itself: |dG - dO|_inf <= 2e-4 |dO|_inf per table, and the tables within 1e-4 of the table maximum.
Row by row the same flip weighs more where a row's terms partly cancel (the flipped term is 2^-8 of itself,
not of the row's sum): per row |dG_r - dO_r|_inf <= 2e-3 |dO_r|_inf (measured <= 3e-4).  Negative ids are
bit-exact.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2005_13789_amd as ne

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def delta_err(before, got, want):
    dg = got.astype(np.float64) - before.astype(np.float64)
    do = want.astype(np.float64) - before.astype(np.float64)
    return np.abs(dg - do).max() / max(np.abs(do).max(), 1e-30)


def rowwise_delta_err(before, got, want):
    """max over rows whose update is not zero of |dG_r - dO_r|_inf / |dO_r|_inf."""
    dg = got.astype(np.float64) - before.astype(np.float64)
    do = want.astype(np.float64) - before.astype(np.float64)
    num, den = np.abs(dg - do).max(axis=1), np.abs(do).max(axis=1)
    live = den > 0
    return float((num[live] / den[live]).max()) if live.any() else 0.0


@pytest.mark.parametrize("V,d,B,N,batches", [(3000, 256, 1000, 256, 3), (2000, 128, 700, 128, 2), (1500, 64, 100, 128, 2),
                                             (5000, 256, 8192, 1024, 1), (900, 256, 1, 128, 1), (4000, 128, 129, 384, 2)])
def test_shared_negative_step(V, d, B, N, batches):
    say(f"shared-negative V={V} d={d} B={B} N={N}")
    rng = np.random.default_rng(V + d + B)
    seed = 11
    deg = (rng.pareto(1.0, V) * 2).astype(np.uint32) + 1
    X = rng.normal(0, 1.5 / np.sqrt(d), (V, d)).astype(np.float32)
    C = rng.normal(0, 1.5 / np.sqrt(d), (V, d)).astype(np.float32)
    vertex = torch.from_numpy(X).to(DEV)
    context = torch.from_numpy(C).to(DEV)
    t = ne.ne_create_tables(vertex, context, seed, init=False)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at)
    ws = torch.empty(ne.ne_shared_workspace_bytes(d, B, N), dtype=torch.uint8, device=DEV)
    neg_dev = torch.empty(N, dtype=torch.int32, device=DEV)
    loss_dev = torch.zeros((), dtype=torch.float64, device=DEV)
    thr, al, _ = oracle.build_alias(deg)
    Xo, Co = X.copy(), C.copy()
    lr, scale = 0.05, 5.0 / N
    for it in range(batches):
        pairs = np.minimum((rng.pareto(0.8, (B, 2)) * V / 50).astype(np.int64), V - 1).astype(np.int32)
        pd = torch.from_numpy(pairs).to(DEV)
        Xb, Cb = Xo.copy(), Co.copy()
        loss_dev.zero_()
        ne.ne_train_batch_shared(t, alias, pd, N, lr, scale, 7 + it, ws, neg_dev, loss_dev)
        torch.cuda.synchronize()
        negs = oracle.sample_shared_negatives(seed, 7 + it, N, thr, al)
        assert np.array_equal(neg_dev.cpu().numpy(), negs)
        loss_o = oracle.train_batch_shared(Xo, Co, pairs, negs, lr, scale, bf16_inputs=True)
        assert abs(loss_dev.item() - loss_o) <= 1e-4 * loss_o, (loss_dev.item(), loss_o)
        Xg, Cg = vertex.cpu().numpy(), context.cpu().numpy()
        ex, ec = delta_err(Xb, Xg, Xo), delta_err(Cb, Cg, Co)
        tx = np.abs(Xg - Xo).max() / np.abs(Xo).max()
        tc = np.abs(Cg - Co).max() / np.abs(Co).max()
        rx, rc = rowwise_delta_err(Xb, Xg, Xo), rowwise_delta_err(Cb, Cg, Co)
        say(f"  batch {it}: delta err X {ex:.2e} C {ec:.2e}; row-wise delta err X {rx:.2e} C {rc:.2e}; table err X {tx:.2e} C {tc:.2e}; loss {loss_o / B:.4f}")
        assert ex <= 2e-4 and ec <= 2e-4
        assert rx <= 2e-3 and rc <= 2e-3
        assert tx <= 1e-4 and tc <= 1e-4
        touched_x = np.zeros(V, bool); touched_x[pairs[:, 0]] = True
        touched_c = np.zeros(V, bool); touched_c[pairs[:, 1]] = True; touched_c[negs] = True
        assert np.array_equal(Xg[~touched_x].view(np.uint32), Xb[~touched_x].view(np.uint32))
        assert np.array_equal(Cg[~touched_c].view(np.uint32), Cb[~touched_c].view(np.uint32))
        # continue both sides from the same state so that errors do not compound across batches
        vertex.copy_(torch.from_numpy(Xo)); context.copy_(torch.from_numpy(Co))


@pytest.mark.parametrize("case", ["all_unique", "one_negative_row", "all_pairs_equal"])
def test_shared_row_sharing_classes(case):
    """Rows named once are rewritten with plain stores, rows named more than once take atomics: the three
    extremes, each from a workspace full of garbage (it needs no initialisation)."""
    say(f"shared-negative row sharing: {case}")
    V, d, B, N = 60000, 128, 2000, 128
    rng = np.random.default_rng(5)
    seed = 3
    if case == "one_negative_row":
        deg = np.zeros(V, np.uint32); deg[77] = 9            # every negative is row 77
    else:
        deg = np.ones(V, np.uint32)
    if case == "all_unique":
        perm = rng.permutation(V).astype(np.int32)
        pairs = np.stack([perm[:B], perm[B:2 * B]], axis=1)  # no row twice among the pairs
    elif case == "one_negative_row":
        pairs = rng.integers(0, V, (B, 2)).astype(np.int32)
        pairs[::7, 1] = 77                                   # the negatives' row is also a positive context
        pairs[::5, 0] = pairs[0, 0]                          # and one source row is named 400 times
    else:
        pairs = np.tile(np.array([[123, 456]], np.int32), (B, 1))
    pairs = np.ascontiguousarray(pairs)
    X = rng.normal(0, 1.5 / np.sqrt(d), (V, d)).astype(np.float32)
    C = rng.normal(0, 1.5 / np.sqrt(d), (V, d)).astype(np.float32)
    vertex, context = torch.from_numpy(X).to(DEV), torch.from_numpy(C).to(DEV)
    t = ne.ne_create_tables(vertex, context, seed, init=False)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at)
    ws = torch.full((ne.ne_shared_workspace_bytes(d, B, N),), 0xFF, dtype=torch.uint8, device=DEV)
    neg_dev = torch.empty(N, dtype=torch.int32, device=DEV)
    thr, al, _ = oracle.build_alias(deg)
    lr, scale = 0.02, 5.0 / N
    Xo, Co = X.copy(), C.copy()
    for it in range(2):                                      # second call: the workspace holds the first call's state
        Xb, Cb = Xo.copy(), Co.copy()
        ne.ne_train_batch_shared(t, alias, torch.from_numpy(pairs).to(DEV), N, lr, scale, it, ws, neg_dev)
        torch.cuda.synchronize()
        negs = oracle.sample_shared_negatives(seed, it, N, thr, al)
        assert np.array_equal(neg_dev.cpu().numpy(), negs)
        if case == "one_negative_row":
            assert (negs == 77).all()
        oracle.train_batch_shared(Xo, Co, pairs, negs, lr, scale, bf16_inputs=True)
        Xg, Cg = vertex.cpu().numpy(), context.cpu().numpy()
        ex, ec = delta_err(Xb, Xg, Xo), delta_err(Cb, Cg, Co)
        say(f"  call {it}: delta err X {ex:.2e} C {ec:.2e}")
        assert ex <= 2e-4 and ec <= 2e-4
        touched_x = np.zeros(V, bool); touched_x[pairs[:, 0]] = True
        touched_c = np.zeros(V, bool); touched_c[pairs[:, 1]] = True; touched_c[negs] = True
        assert np.array_equal(Xg[~touched_x].view(np.uint32), Xb[~touched_x].view(np.uint32))
        assert np.array_equal(Cg[~touched_c].view(np.uint32), Cb[~touched_c].view(np.uint32))
        vertex.copy_(torch.from_numpy(Xo)); context.copy_(torch.from_numpy(Co))


def test_shared_argument_errors():
    V, d = 500, 128
    vertex = torch.zeros((V, d), dtype=torch.float32, device=DEV)
    context = torch.zeros((V, d), dtype=torch.float32, device=DEV)
    t = ne.ne_create_tables(vertex, context, 0, init=False)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(np.ones(V, np.uint32), 0, at)
    pairs = torch.zeros((16, 2), dtype=torch.int32, device=DEV)
    ws = torch.empty(ne.ne_shared_workspace_bytes(d, 16, 128), dtype=torch.uint8, device=DEV)
    assert ne.ne_shared_workspace_bytes(d, 16, 100) == 0 and ne.ne_shared_workspace_bytes(96, 16, 128) == 0
    with pytest.raises(ne.NeError):
        ne.ne_train_batch_shared(t, alias, pairs, 100, 0.1, 0.1, 0, ws)          # N not a multiple of 128
    with pytest.raises(ne.NeError):
        ne.ne_train_batch_shared(t, alias, pairs, 256, 0.1, 0.1, 0, ws)          # workspace too small
    with pytest.raises(ne.NeError):
        ne.ne_train_batch_shared(t, alias, pairs, 128, float("inf"), 0.1, 0, ws)
    ne.ne_train_batch_shared(t, alias, pairs[:0], 128, 0.1, 0.1, 0, ws)          # empty batch: no-op
    torch.cuda.synchronize()
    assert not vertex.any() and not context.any()
