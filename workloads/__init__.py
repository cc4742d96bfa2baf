"""Seeded synthetic inputs for SGNS node-embedding training.

The paper trains on social / web graphs (YouTube, Hyperlink-PLD, Friendster, kron, delaunay and
internal or generated networks, Table II) that are not available here.  R-MAT graphs stand in for
them: kron is itself a Kronecker/R-MAT graph, and the generated networks are said to resemble
social-network topology, i.e. a skewed degree distribution, which is what drives row reuse and
atomic contention in the training kernels.

This module holds input generation only: graphs, degrees, random walks, the (src, ctx) pairs cut
from them (Algorithm 1, network augmentation), shuffling and the 2-D bucketing of pairs into
(src-block, ctx-block) sample blocks (Sec. III-A).  It contains none of the method's arithmetic and is
the only code that both the CPU oracle's tests and the GPU path's tests use.  Everything is written
with torch tensor ops so the same recipe runs on the CPU (small cases) and on the GPU (the 100 M-node
cases, where a host generator would take many minutes).  A torch.Generator seeded per call makes each
recipe reproducible on a given device type.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _scramble_params(V: int):
    """Multiplier/offset of the affine bijection id -> (id*A + Bc) mod V (A coprime to V)."""
    A = 2654435761 % V
    if A < 2:
        A = 1
    while math.gcd(A, V) != 1:
        A += 1
    Bc = 40503 % V
    return A, Bc


def rmat_edges(V: int, n_edges: int, seed: int, abc=(0.57, 0.19, 0.19), device="cpu",
               scramble: bool = True) -> torch.Tensor:
    """int64[n_edges][2] directed R-MAT edges over ids [0, V).

    Recursive quadrant choice with probabilities (a, b, c, 1-a-b-c) over ceil(log2 V) levels, no
    parameter noise; ids >= V are rejected and redrawn; ids then go through a fixed affine bijection
    of [0, V) so that hubs are spread over id blocks (the paper balances partitions by degree).
    Self-loops and duplicates are kept here; callers that build a graph drop self-loops.
    """
    a, b, c = abc
    scale = max(1, math.ceil(math.log2(V)))
    g = _gen(seed, device)
    out = torch.empty((n_edges, 2), dtype=torch.int64, device=device)
    todo = torch.arange(n_edges, device=device)
    while todo.numel() > 0:
        n = todo.numel()
        src = torch.zeros(n, dtype=torch.int64, device=device)
        dst = torch.zeros(n, dtype=torch.int64, device=device)
        for _ in range(scale):
            r = torch.rand(n, generator=g, device=device)
            sbit = (r >= a + b).to(torch.int64)
            dbit = (((r >= a) & (r < a + b)) | (r >= a + b + c)).to(torch.int64)
            src = src * 2 + sbit
            dst = dst * 2 + dbit
        ok = (src < V) & (dst < V)
        out[todo[ok], 0] = src[ok]
        out[todo[ok], 1] = dst[ok]
        todo = todo[~ok]
    if scramble:
        A, Bc = _scramble_params(V)
        out = (out * A + Bc) % V
    return out


@dataclass
class Graph:
    """Symmetrised multigraph in CSR form.  degree[i] = number of edge endpoints at node i."""
    num_nodes: int
    indptr: torch.Tensor    # int64[V+1]
    indices: torch.Tensor   # int64[2*E']
    degree: torch.Tensor    # int64[V]


def build_graph(V: int, edges: torch.Tensor) -> Graph:
    """Drop self-loops, add the reverse of every edge (multi-edges kept), build CSR."""
    keep = edges[:, 0] != edges[:, 1]
    e = edges[keep]
    src = torch.cat([e[:, 0], e[:, 1]])
    dst = torch.cat([e[:, 1], e[:, 0]])
    order = torch.argsort(src, stable=True)
    src, dst = _take_rows(src, order), _take_rows(dst, order)
    degree = torch.bincount(src, minlength=V)
    indptr = torch.zeros(V + 1, dtype=torch.int64, device=edges.device)
    indptr[1:] = torch.cumsum(degree, 0)
    return Graph(V, indptr, dst, degree)


def rmat_degrees(V: int, n_edges: int, seed: int, abc=(0.57, 0.19, 0.19), device="cpu",
                 chunk: int = 1 << 25) -> torch.Tensor:
    """int64[V] endpoint counts of a symmetrised R-MAT graph, streamed in chunks (graph not kept)."""
    deg = torch.zeros(V, dtype=torch.int64, device=device)
    done = 0
    part = 0
    while done < n_edges:
        n = min(chunk, n_edges - done)
        e = rmat_edges(V, n, seed * 1000003 + part, abc, device)
        keep = e[:, 0] != e[:, 1]
        deg += torch.bincount(e[keep].reshape(-1), minlength=V)
        done += n
        part += 1
    return deg


def _take_rows(t: torch.Tensor, index: torch.Tensor, chunk: int = 1 << 24) -> torch.Tensor:
    """t[index] for a 1-D index of any length, gathered a bounded number of rows at a time (one indexing
    call over 2^26 rows of a two-column tensor fails to launch on this PyTorch build and leaves its output
    unwritten)."""
    if index.numel() <= chunk:
        return t[index]
    out = torch.empty((index.numel(),) + tuple(t.shape[1:]), dtype=t.dtype, device=t.device)
    for lo in range(0, index.numel(), chunk):
        out[lo:lo + chunk] = t[index[lo:lo + chunk]]
    return out


def random_walks(graph: Graph, starts: torch.Tensor, length: int, seed: int) -> torch.Tensor:
    """int64[len(starts)][length] uniform random walks (length counts nodes, not steps)."""
    dev = starts.device
    g = _gen(seed, dev)
    walks = torch.empty((starts.numel(), length), dtype=torch.int64, device=dev)
    cur = starts.clone()
    walks[:, 0] = cur
    for t in range(1, length):
        lo = graph.indptr[cur]
        deg = graph.indptr[cur + 1] - lo
        pick = (torch.rand(cur.numel(), generator=g, device=dev, dtype=torch.float64) * deg).to(torch.int64)
        pick = torch.minimum(pick, deg - 1)
        cur = graph.indices[lo + pick]
        walks[:, t] = cur
    return walks


def walk_pairs(graph: Graph, length: int, window: int, n_pairs: int | None, seed: int) -> torch.Tensor:
    """int32[n][2] shuffled positive (src, ctx) pairs from random walks.

    Algorithm 1 (network augmentation): every node v starts a walk and each node u that follows v on
    the walk within `window` positions gives a sample (v, u); the earlier node is the source.  One
    walk per non-isolated node.  When n_pairs is smaller than what all walks give, only as many
    uniformly chosen start nodes are walked as are needed (instead of generating everything and
    truncating after the shuffle), then the pairs are shuffled and cut to n_pairs.
    """
    dev = graph.degree.device
    g = _gen(seed + 7919, dev)
    starts = torch.nonzero(graph.degree > 0).reshape(-1)
    per_walk = sum(length - j for j in range(1, window + 1) if length - j > 0)
    if n_pairs is not None and per_walk > 0:
        need = -(-n_pairs // per_walk)
        if need < starts.numel():
            sel = torch.randperm(starts.numel(), generator=g, device=dev)[:need]
            starts = starts[sel]
    walks = random_walks(graph, starts, length, seed)
    parts = []
    for j in range(1, window + 1):
        if length - j <= 0:
            break
        parts.append(torch.stack([walks[:, :-j].reshape(-1), walks[:, j:].reshape(-1)], dim=1))
    pairs = torch.cat(parts)
    perm = torch.randperm(pairs.shape[0], generator=g, device=dev)
    pairs = _take_rows(pairs, perm)
    if n_pairs is not None:
        pairs = pairs[:n_pairs]
    return pairs.to(torch.int32).contiguous()


def rmat_pairs(V: int, n_pairs: int, seed: int, abc=(0.57, 0.19, 0.19), device="cpu",
               chunk: int = 1 << 25) -> torch.Tensor:
    """int32[n_pairs][2] positive pairs drawn directly as R-MAT edges (both directions equally likely).

    Stand-in for walk pairs on graphs too large to walk on the host: a walk visits nodes in proportion
    to degree, and so do the endpoints of R-MAT edges.  Self-pairs are dropped and redrawn.
    """
    out = torch.empty((n_pairs, 2), dtype=torch.int32, device=device)
    done = 0
    part = 0
    g = _gen(seed + 104729, device)
    while done < n_pairs:
        n = min(chunk, n_pairs - done)
        e = rmat_edges(V, n + n // 64 + 16, seed * 1000003 + 500009 + part, abc, device)
        e = e[e[:, 0] != e[:, 1]][:n]
        flip = torch.rand(e.shape[0], generator=g, device=device) < 0.5
        e = torch.where(flip[:, None], e.flip(1), e)
        out[done:done + e.shape[0]] = e.to(torch.int32)
        done += e.shape[0]
        part += 1
    return out


@dataclass
class BucketedPairs:
    """Pairs grouped into grid x grid (src-block, ctx-block) sample blocks (2-D partitioning)."""
    pairs: torch.Tensor        # int32[n][2], sorted by bucket id = src_block*grid + ctx_block
    offsets: torch.Tensor      # int64[grid*grid + 1] (host)
    grid: int
    block_rows: int


def bucket_pairs(pairs: torch.Tensor, V: int, grid: int) -> BucketedPairs:
    """Group pairs by (src // block_rows, ctx // block_rows), keeping their order inside a bucket."""
    block_rows = -(-V // grid)
    p = pairs.to(torch.int64)
    bid = (p[:, 0] // block_rows) * grid + (p[:, 1] // block_rows)
    order = torch.argsort(bid, stable=True)
    counts = torch.bincount(bid, minlength=grid * grid).cpu()
    offsets = torch.zeros(grid * grid + 1, dtype=torch.int64)
    offsets[1:] = torch.cumsum(counts, 0)
    return BucketedPairs(_take_rows(pairs, order).contiguous(), offsets, grid, block_rows)


def orthogonal_schedule(bp: BucketedPairs, batch: int):
    """List of (start, count, src_block, ctx_block) batches.

    Buckets are visited in the orthogonal-block order of one GPU group (Sec. III-B): for shift e, for
    i: bucket (i, (i+e) mod grid).  Batches never straddle a bucket; a bucket's last batch may be short.
    """
    sched = []
    gsz = bp.grid
    for e in range(gsz):
        for i in range(gsz):
            j = (i + e) % gsz
            lo = int(bp.offsets[i * gsz + j])
            hi = int(bp.offsets[i * gsz + j + 1])
            s = lo
            while s < hi:
                n = min(batch, hi - s)
                sched.append((s, n, i, j))
                s += n
    return sched


def linear_decay_lr(lr0: float, pairs_done: int, pairs_total: int) -> float:
    """lr_t = lr0 * max(1 - done/total, 1e-4), computed in fp64 by the caller of the library."""
    return lr0 * max(1.0 - pairs_done / pairs_total, 1e-4)
