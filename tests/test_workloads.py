"""Host checks of the synthetic input recipes (no method arithmetic involved)."""
import numpy as np
import torch

import workloads as wl


def test_rmat_graph_and_walk_pairs_small():
    V, E = 2000, 20000
    e = wl.rmat_edges(V, E, seed=0)
    assert e.shape == (E, 2) and e.min() >= 0 and e.max() < V
    assert torch.equal(e, wl.rmat_edges(V, E, seed=0))
    g = wl.build_graph(V, e)
    assert int(g.degree.sum()) == g.indices.numel() == int(g.indptr[-1])
    # skewed: the top 1% of nodes hold far more than 1% of the endpoints
    top = torch.sort(g.degree, descending=True).values[: V // 100].sum().item()
    assert top > 0.08 * g.degree.sum().item()
    L, w = 40, 5
    pairs = wl.walk_pairs(g, L, w, None, seed=0)
    n_start = int((g.degree > 0).sum())
    assert pairs.shape[0] == n_start * sum(L - j for j in range(1, w + 1))
    assert pairs.dtype == torch.int32
    # every pair's endpoints are non-isolated nodes; consecutive-step pairs are real edges
    walks = wl.random_walks(g, torch.nonzero(g.degree > 0).reshape(-1)[:50], 10, seed=3)
    for row in walks.tolist():
        for a, b in zip(row[:-1], row[1:]):
            nb = g.indices[g.indptr[a]:g.indptr[a + 1]].tolist()
            assert b in nb
    few = wl.walk_pairs(g, L, w, 5000, seed=0)
    assert few.shape == (5000, 2)


def test_bucketing_and_schedule():
    V, grid, B = 1000, 4, 64
    pairs = wl.rmat_pairs(V, 20000, seed=2)
    assert (pairs[:, 0] != pairs[:, 1]).all()
    bp = wl.bucket_pairs(pairs, V, grid)
    assert int(bp.offsets[-1]) == pairs.shape[0]
    sched = wl.orthogonal_schedule(bp, B)
    assert sum(n for _, n, _, _ in sched) == pairs.shape[0]
    p = bp.pairs.numpy()
    seen = set()
    for s, n, i, j in sched:
        blk = p[s:s + n]
        assert n <= B
        assert ((blk[:, 0] // bp.block_rows) == i).all() and ((blk[:, 1] // bp.block_rows) == j).all()
        seen.add((i, j))
    assert len(seen) == grid * grid
    # within one shift e the src blocks and the ctx blocks are all distinct (orthogonal blocks)
    order = []
    for _, _, i, j in sched:
        if not order or order[-1] != (i, j):
            order.append((i, j))
    for e in range(grid):
        grp = order[e * grid:(e + 1) * grid]
        assert len({i for i, _ in grp}) == grid and len({j for _, j in grp}) == grid


def test_degrees_streamed_equals_graph_degrees_in_distribution():
    V = 5000
    d1 = wl.rmat_degrees(V, 40000, seed=1, chunk=10000)
    assert d1.shape == (V,) and int(d1.sum()) <= 80000 and int(d1.sum()) > 70000
    assert wl.linear_decay_lr(0.025, 0, 100) == 0.025
    assert wl.linear_decay_lr(0.025, 100, 100) == 0.025 * 1e-4


def test_take_rows_in_chunks_equals_plain_indexing():
    """Large gathers go through _take_rows a bounded number of rows at a time; any chunk size gives t[index]."""
    g = torch.Generator().manual_seed(3)
    t = torch.randint(0, 1000, (5000, 2), generator=g)
    index = torch.randperm(5000, generator=g)
    for chunk in (1, 7, 4999, 5000, 1 << 24):
        assert torch.equal(wl._take_rows(t, index, chunk), t[index])
    v = torch.arange(100)
    assert torch.equal(wl._take_rows(v, torch.tensor([5, 1, 99]), 2), torch.tensor([5, 1, 99]))
