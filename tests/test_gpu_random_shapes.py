"""Seeded random shapes: for 40 draws of (nodes, dim, K, batch, number of batches, id skew) the exact step -
through ne_train_batch, ne_train_block (ragged last batch) and ne_train_walks - is compared with the oracle
element by element.  The shapes mix every launch shape (dim 4 .. 1024, K 0 .. 62), batches far below and above a
workgroup's share, and id distributions from "every row once" to "two rows take everything"."""
import numpy as np
import pytest
import torch

import oracle
import paper_2005_13789_amd as ne
from parity_util import rowwise_rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def draw_case(i):
    rng = np.random.default_rng(1000 + i)
    d = int(rng.choice([4, 8, 12, 32, 64, 100, 128, 200, 256, 384, 512, 1000, 1024]))
    # lanes per pair grow with K; keep the work of a case small when rows are wide
    K = int(rng.choice([0, 1, 2, 5, 5, 10, 15, 30, 62]))
    budget = 600_000 // (d * (K + 2))
    B = int(np.clip(rng.integers(1, 3000), 1, max(budget, 1)))
    V = int(rng.choice([7, 50, 1000, 20000]))
    nb = int(rng.integers(1, 4))
    skew = str(rng.choice(["uniform", "pareto", "two_rows", "distinct"]))
    return rng, V, d, K, B, nb, skew


def ids(rng, skew, V, shape):
    if skew == "uniform":
        return rng.integers(0, V, shape).astype(np.int32)
    if skew == "pareto":
        return ((rng.pareto(0.8, shape) * V / 20).astype(np.int64) % V).astype(np.int32)
    if skew == "two_rows":
        return rng.integers(0, min(V, 2), shape).astype(np.int32)
    n = int(np.prod(shape))                                   # distinct while the table lasts
    return (np.arange(n) % V).reshape(shape).astype(np.int32)


def tables(V, d, max_B, K, seed, rng):
    vertex = torch.from_numpy(rng.normal(0, 1.0 / np.sqrt(d), (V, d)).astype(np.float32)).to(DEV)
    context = torch.from_numpy(rng.normal(0, 1.0 / np.sqrt(d), (V, d)).astype(np.float32)).to(DEV)
    ws = torch.empty(ne.ne_workspace_bytes(d, max_B, K), dtype=torch.uint8, device=DEV)
    return ne.ne_create_tables(vertex, context, seed, init=False, max_batch=max_B, max_negatives=K, workspace=ws)


@pytest.mark.parametrize("i", range(40))
def test_random_shape(i):
    rng, V, d, K, B, nb, skew = draw_case(i)
    seed, base = 77 + i, int(rng.integers(0, 2**40))
    say(f"case {i}: V={V} d={d} K={K} B={B} batches={nb} ids={skew}")
    deg = (rng.pareto(1.0, V) * 2).astype(np.uint32) + 1
    thr, al, _ = oracle.build_alias(deg)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at) if K > 0 else None
    n_pairs = nb * B - int(rng.integers(0, B))                # ragged last batch
    pairs = ids(rng, skew, V, (n_pairs, 2))
    lrs = [0.03 / (1 + b) for b in range(nb)]
    tol = 1e-4 * nb

    # pairs: ne_train_block on one handle, ne_train_batch batch by batch on another
    tb, t1 = tables(V, d, B, K, seed, np.random.default_rng(i)), tables(V, d, B, K, seed, np.random.default_rng(i))
    Xo, Co = tb.vertex.cpu().numpy(), tb.context.cpu().numpy()
    neg_dev = torch.empty((n_pairs, max(K, 1)), dtype=torch.int32, device=DEV)
    pd = torch.from_numpy(pairs).to(DEV)
    ne.ne_train_block(tb, alias, pd, B, K, lrs, base, neg_dev if K > 0 else None)
    for b in range(nb):
        ne.ne_train_batch(t1, alias, pd[b * B:(b + 1) * B], K, lrs[b], base + b * B)
    torch.cuda.synchronize()
    neg = oracle.sample_negatives(seed, base, n_pairs, K, thr, al)
    if K > 0:
        assert np.array_equal(neg_dev.cpu().numpy(), neg)
    for b in range(nb):
        sl = slice(b * B, min((b + 1) * B, n_pairs))
        oracle.train_batch(Xo, Co, np.ascontiguousarray(pairs[sl]), np.ascontiguousarray(neg[sl]), lrs[b])
    for name, t in (("block", tb), ("batch", t1)):
        ex = rowwise_rel_err(t.vertex.cpu().numpy(), Xo)
        ec = rowwise_rel_err(t.context.cpu().numpy(), Co)
        assert ex <= tol and ec <= tol, (name, ex, ec)

    # walks of the same shape family
    L = int(rng.integers(2, 24))
    window = int(rng.integers(1, min(L, 9)))
    R = 1 + window * (K + 1)
    wpb = max(1, min(B, 600_000 // (d * R * L)))
    n_walks = nb * wpb - int(rng.integers(0, wpb))
    walks = ids(rng, skew, V, (n_walks, L))
    walks[rng.random((n_walks, L)) < 0.1] = -1
    tw = tables(V, d, -(-(wpb * L * R) // (K + 2)), K, seed, np.random.default_rng(i))
    Xo, Co = tw.vertex.cpu().numpy(), tw.context.cpu().numpy()
    ne.ne_train_walks(tw, alias, torch.from_numpy(walks).to(DEV), wpb, window, K, lrs, base)
    torch.cuda.synchronize()
    for b in range(nb):
        part = np.ascontiguousarray(walks[b * wpb:(b + 1) * wpb])
        if part.shape[0] == 0:
            continue
        wp, sample = oracle.walk_pairs(part, window)
        first = b * wpb * L * window
        neg_all = oracle.sample_negatives(seed, base + first, part.shape[0] * L * window, K, thr, al)
        oracle.train_batch(Xo, Co, wp, np.ascontiguousarray(neg_all[sample]), lrs[b])
    ex = rowwise_rel_err(tw.vertex.cpu().numpy(), Xo)
    ec = rowwise_rel_err(tw.context.cpu().numpy(), Co)
    assert ex <= tol and ec <= tol, ("walks", ex, ec)
