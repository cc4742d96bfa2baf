"""Link-prediction evaluation of trained embeddings (Sec. V-B "Link Prediction").

The protocol of the paper's evaluation: the edges of a network are split into a training set and a
held-out test set; embeddings are trained on walks over the training edges only (negatives drawn
during training); the test set is scored together with the same number of random node pairs that are
not edges of the network, and the result is the AUC of that ranking.

The paper does not say which score ranks a pair.  Reading taken here: the model's own similarity
score, vertex[u] . context[v] (`second_from_context=True`, what training maximises for observed pairs);
vertex[u] . vertex[v] is available as the alternative.  Scores come from the library's
`ne_score_pairs`; the split, the non-edge sampling and the AUC are host-side bookkeeping on small
arrays and use numpy.

The paper evaluates on YouTube and Hyperlink-PLD; neither ships here, so `read_edge_list` takes any
"u v" text file a user supplies and the tests use a synthetic planted-partition network.
"""
from __future__ import annotations

import numpy as np
import torch

import paper_2005_13789_amd as ne
import workloads as wl


def read_edge_list(path: str):
    """Edges of a whitespace-separated "u v" text file (lines starting with # or % are comments).

    Returns (int64[E][2] with ids renumbered densely in order of first appearance, number of nodes).
    """
    raw = np.loadtxt(path, dtype=np.int64, comments=("#", "%"), usecols=(0, 1), ndmin=2)
    ids, first, inverse = np.unique(raw.reshape(-1), return_index=True, return_inverse=True)
    order = np.argsort(np.argsort(first))            # rank of each distinct id by first appearance
    return order[inverse].reshape(-1, 2), int(ids.size)


def split_edges(edges: np.ndarray, test_fraction: float, seed: int):
    """Random split of the edge list into (train, test); duplicates and self-loops are dropped first and an
    undirected edge appears once, as (min, max)."""
    e = np.sort(np.asarray(edges, dtype=np.int64), axis=1)
    e = e[e[:, 0] != e[:, 1]]
    e = np.unique(e, axis=0)
    rng = np.random.default_rng(seed)
    perm = rng.permutation(e.shape[0])
    n_test = max(1, int(round(test_fraction * e.shape[0])))
    return e[perm[n_test:]], e[perm[:n_test]]


def sample_non_edges(num_nodes: int, edges: np.ndarray, n: int, seed: int) -> np.ndarray:
    """int64[n][2] random node pairs that are neither self-pairs nor edges of the network (either direction)."""
    e = np.sort(np.asarray(edges, dtype=np.int64), axis=1)
    keys = np.unique(e[:, 0] * num_nodes + e[:, 1])
    rng = np.random.default_rng(seed)
    out = np.empty((0, 2), dtype=np.int64)
    while out.shape[0] < n:
        cand = rng.integers(0, num_nodes, (2 * (n - out.shape[0]) + 16, 2))
        lo, hi = cand.min(axis=1), cand.max(axis=1)
        k = lo * num_nodes + hi
        pos = np.searchsorted(keys, k)
        is_edge = (pos < keys.size) & (keys[np.minimum(pos, keys.size - 1)] == k)
        out = np.concatenate([out, cand[(lo != hi) & ~is_edge]])
    return out[:n]


def auc(pos_scores: np.ndarray, neg_scores: np.ndarray) -> float:
    """Probability that a random positive outranks a random negative, ties counting one half
    (the Mann-Whitney statistic from average ranks)."""
    pos = np.asarray(pos_scores, dtype=np.float64)
    neg = np.asarray(neg_scores, dtype=np.float64)
    allv = np.concatenate([pos, neg])
    order = np.argsort(allv, kind="mergesort")
    sorted_v = allv[order]
    ranks = np.empty(allv.size, dtype=np.float64)
    # average rank over runs of equal values
    boundaries = np.flatnonzero(np.concatenate([[True], sorted_v[1:] != sorted_v[:-1], [True]]))
    for a, b in zip(boundaries[:-1], boundaries[1:]):
        ranks[order[a:b]] = 0.5 * (a + b - 1) + 1.0
    u = ranks[:pos.size].sum() - pos.size * (pos.size + 1) / 2.0
    return float(u / (pos.size * neg.size))


def score(tables: ne.Tables, pairs: np.ndarray, second_from_context: bool = True) -> np.ndarray:
    """Scores of int pairs [n][2] at the current tables (float32[n], host)."""
    dev = tables.vertex.device
    p = torch.from_numpy(np.ascontiguousarray(pairs, dtype=np.int32)).to(dev)
    s = torch.empty(p.shape[0], dtype=torch.float32, device=dev)
    ne.ne_score_pairs(tables, p, s, second_from_context)
    return s.cpu().numpy()


def evaluate(tables: ne.Tables, num_nodes: int, all_edges: np.ndarray, test_edges: np.ndarray, seed: int,
             second_from_context: bool = True) -> float:
    """AUC of the held-out edges against as many random non-edges of the whole network."""
    negatives = sample_non_edges(num_nodes, all_edges, test_edges.shape[0], seed)
    return auc(score(tables, test_edges, second_from_context), score(tables, negatives, second_from_context))


def train(train_edges: np.ndarray, num_nodes: int, dim: int = 64, epochs: int = 3, negatives: int = 5,
          batch: int = 4096, lr0: float = 0.025, walk_length: int = 40, window: int = 5, seed: int = 0,
          mode: str = "sync", device: str = "cuda:0"):
    """Embeddings from walks over the training edges: per epoch one walk per node, window pairs shuffled,
    batches of `batch` pairs through ne_train_block (mode "sync", the exact step) or ne_train_block_async
    (mode "async", the per-sample mode), or the walks themselves through ne_train_walks (mode "walks": the exact step on batches of
    whole walks, unshuffled), learning rate decaying linearly over the run.  Returns (Tables, Alias); the handles keep
    their device tensors alive (tables.vertex, tables.context)."""
    dev = torch.device(device)
    graph = wl.build_graph(num_nodes, torch.from_numpy(np.asarray(train_edges, dtype=np.int64)))
    vertex = torch.empty((num_nodes, dim), dtype=torch.float32, device=dev)
    context = torch.empty((num_nodes, dim), dtype=torch.float32, device=dev)
    max_batch = batch
    if mode == "walks":      # references of a batch of whole walks: entries x (1 + window (K + 1))
        per_walk = sum(walk_length - j for j in range(1, window + 1) if walk_length - j > 0)
        refs = max(1, batch // max(per_walk, 1)) * walk_length * (1 + window * (negatives + 1))
        max_batch = max(batch, -(-refs // (negatives + 2)))
    ws = torch.empty(ne.ne_workspace_bytes(dim, max_batch, negatives), dtype=torch.uint8, device=dev)
    tables = ne.ne_create_tables(vertex, context, seed, init=True, max_batch=max_batch, max_negatives=negatives, workspace=ws)
    table = torch.empty((num_nodes, 2), dtype=torch.int32, device=dev)
    alias = ne.ne_build_neg_alias(graph.degree.clamp(max=2**32 - 1).numpy().astype(np.uint32), 0, table)
    if mode == "walks":
        # on-device augmentation: the walks themselves are the input; a batch is as many whole walks as hold
        # about `batch` samples
        per_walk = sum(walk_length - j for j in range(1, window + 1) if walk_length - j > 0)
        wpb = max(1, batch // max(per_walk, 1))
        starts = torch.nonzero(graph.degree > 0).reshape(-1)
        gen = torch.Generator().manual_seed(seed)
        n_batches = -(-starts.numel() // wpb)
        for e in range(epochs):
            order = starts[torch.randperm(starts.numel(), generator=gen)]
            walks = wl.random_walks(graph, order, walk_length, seed + 1 + e).to(torch.int32).to(dev).contiguous()
            lrs = np.array([wl.linear_decay_lr(lr0, e * n_batches + b, epochs * n_batches) for b in range(n_batches)],
                           dtype=np.float32)
            ne.ne_train_walks(tables, alias, walks, wpb, window, negatives, lrs,
                              e * starts.numel() * walk_length * window)
        torch.cuda.synchronize(dev)
        return tables, alias
    epoch_pairs = [wl.walk_pairs(graph, walk_length, window, None, seed + 1 + e) for e in range(epochs)]
    total = sum(int(p.shape[0]) for p in epoch_pairs)
    done = 0
    for pairs in epoch_pairs:
        p = pairs.to(torch.int32).to(dev).contiguous()
        n = int(p.shape[0])
        starts = list(range(0, n, batch))
        lrs = np.array([wl.linear_decay_lr(lr0, done + s, total) for s in starts], dtype=np.float32)
        if mode == "sync":
            ne.ne_train_block(tables, alias, p, batch, negatives, lrs, done)
        elif mode == "async":
            ne.ne_train_block_async(tables, alias, p, batch, negatives, lrs, done)
        else:
            raise ValueError("mode must be 'sync', 'async' or 'walks'")
        done += n
    torch.cuda.synchronize(dev)
    return tables, alias


def main(argv=None) -> int:
    """python -m paper_2005_13789_amd.linkpred EDGES.txt [options]: split, train, report the AUC."""
    import argparse
    import json
    ap = argparse.ArgumentParser(description="Link-prediction AUC of SGNS embeddings trained on an edge list (Sec. V-B protocol)")
    ap.add_argument("edges", help='text file with one "u v" edge per line (# and % start comments)')
    ap.add_argument("--test-fraction", type=float, default=0.01, help="share of the edges held out (the paper: 1 %% on YouTube)")
    ap.add_argument("--dim", type=int, default=128)
    ap.add_argument("--epochs", type=int, default=10)
    ap.add_argument("--negatives", type=int, default=5)
    ap.add_argument("--batch", type=int, default=65536)
    ap.add_argument("--lr", type=float, default=0.025)
    ap.add_argument("--walk-length", type=int, default=40)
    ap.add_argument("--window", type=int, default=5)
    ap.add_argument("--mode", default="sync", choices=["sync", "walks", "async"])
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args(argv)
    edges, n = read_edge_list(args.edges)
    train_edges, test_edges = split_edges(edges, args.test_fraction, args.seed)
    tables, _alias = train(train_edges, n, dim=args.dim, epochs=args.epochs, negatives=args.negatives, batch=args.batch,
                           lr0=args.lr, walk_length=args.walk_length, window=args.window, seed=args.seed, mode=args.mode)
    all_edges = np.concatenate([train_edges, test_edges])
    print(json.dumps({"nodes": n, "train_edges": int(train_edges.shape[0]), "test_edges": int(test_edges.shape[0]),
                      "auc_vertex_context": evaluate(tables, n, all_edges, test_edges, args.seed + 1, True),
                      "auc_vertex_vertex": evaluate(tables, n, all_edges, test_edges, args.seed + 1, False)}))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
