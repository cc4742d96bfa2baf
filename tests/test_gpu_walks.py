"""ne_train_walks (on-device augmentation, Algorithm 1) against the oracle: the oracle expands the walks into
samples, draws the negatives for the same sample indices and runs its minibatch step batch by batch; the GPU
trains on the walks directly.  Negatives bit-exact, tables to the 1e-4 row-wise bar, untouched rows bit-identical,
and the same result as ne_train_block on the expanded pairs when the indices agree."""
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


def make(V, d, max_B, max_K, seed):
    vertex = torch.empty((V, d), dtype=torch.float32, device=DEV)
    context = torch.empty((V, d), dtype=torch.float32, device=DEV)
    ws = torch.empty(ne.ne_workspace_bytes(d, max_B, max_K), dtype=torch.uint8, device=DEV)
    t = ne.ne_create_tables(vertex, context, seed, init=True, max_batch=max_B, max_negatives=max_K, workspace=ws)
    context.copy_(torch.randn((V, d), generator=torch.Generator().manual_seed(seed)).to(DEV) * 0.1)
    return t


def oracle_run(X, C, walks, wpb, window, K, lrs, seed, sample_base, thr, al, base=0):
    """The oracle's result of the same call, and the negatives it drew per existing sample."""
    n, L = walks.shape
    negs_by_sample = {}
    for b, first in enumerate(range(0, n, wpb)):
        part = np.ascontiguousarray(walks[first:first + wpb])
        pairs, sample = oracle.walk_pairs(part, window)
        sample = sample + first * L * window
        span = part.shape[0] * L * window
        neg_all = oracle.sample_negatives(seed, sample_base + first * L * window, span, K, thr, al, base)
        neg = np.ascontiguousarray(neg_all[sample - first * L * window])
        for s, row in zip(sample, neg):
            negs_by_sample[int(s)] = row
        oracle.train_batch(X, C, pairs, neg, lrs[b])
    return negs_by_sample


@pytest.mark.parametrize("V,d,K,n,L,window,wpb", [
    (5000, 128, 5, 60, 40, 5, 20),       # three batches
    (300, 64, 3, 25, 12, 4, 7),          # small graph: almost every row shared; ragged last batch
    (4000, 512, 10, 10, 20, 10, 10),     # wide rows, window = half the walk
    (2000, 32, 0, 30, 9, 2, 30),         # no negatives
    (800, 256, 62, 3, 6, 1, 3),          # the most negatives, window 1
    (100000, 128, 5, 170, 80, 5, 170),   # the shape of config 2: one batch of 170 walks, 65450 samples
    # walk lengths that fill whole segments of a workgroup's entries: the train kernel then works by segments
    (5000, 128, 5, 60, 48, 5, 20),
    (300, 64, 3, 25, 32, 4, 7),          # small graph, segments, nearly every row shared
    (2000, 32, 0, 30, 64, 2, 30),        # segments without negatives
    (50000, 128, 5, 40, 80, 14, 40),     # window = entries per segment - 2, the widest that still goes by segments
    (700, 128, 1, 9, 33, 3, 4),          # one entry past a segment boundary
])
def test_walks_match_oracle(V, d, K, n, L, window, wpb):
    say(f"walks V={V} d={d} K={K} n={n} L={L} window={window} per batch={wpb}")
    rng = np.random.default_rng(V + n + L)
    seed, sample_base = 21, 1000
    deg = (rng.pareto(1.0, V) * 3).astype(np.uint32) + 1
    walks = ((rng.pareto(0.9, (n, L)) * V / 30).astype(np.int64) % V).astype(np.int32)
    # short walks (padded), a hole in the middle of one, and an empty walk
    for r in range(0, n, 4):
        walks[r, rng.integers(1, L):] = -1
    if n > 2:
        walks[1, L // 2] = -1
        walks[2, :] = -1
    R = 1 + window * (K + 1)
    max_B = -(-(wpb * L * R) // (K + 2))
    t = make(V, d, max_B, K, seed)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at) if K > 0 else None
    thr, al, _ = oracle.build_alias(deg)
    n_batches = -(-n // wpb)
    lrs = [0.02 / (1 + b) for b in range(n_batches)]
    Xo, Co = t.vertex.cpu().numpy(), t.context.cpu().numpy()
    Xb, Cb = Xo.copy(), Co.copy()
    neg_out = torch.full((n, L, window, max(K, 1)), -7, dtype=torch.int32, device=DEV)
    ne.ne_train_walks(t, alias, torch.from_numpy(walks).to(DEV), wpb, window, K, lrs, sample_base, neg_out if K > 0 else None)
    torch.cuda.synchronize()
    negs = oracle_run(Xo, Co, walks, wpb, window, K, lrs, seed, sample_base, thr, al)
    if K > 0:
        got = neg_out.cpu().numpy().reshape(n * L * window, K)
        exists = np.zeros(n * L * window, bool)
        for s, row in negs.items():
            exists[s] = True
            assert np.array_equal(got[s], row), f"negatives of sample {s}"
        assert np.all(got[~exists] == -7)                     # rows of samples that do not exist are untouched
    Xg, Cg = t.vertex.cpu().numpy(), t.context.cpu().numpy()
    ex, ec = rowwise_rel_err(Xg, Xo), rowwise_rel_err(Cg, Co)
    say(f"  {len(negs)} samples; row error X {ex:.2e} C {ec:.2e}")
    assert ex <= 1e-4 * n_batches and ec <= 1e-4 * n_batches
    same_x = np.all(Xo.view(np.uint32) == Xb.view(np.uint32), axis=1)
    same_c = np.all(Co.view(np.uint32) == Cb.view(np.uint32), axis=1)
    pairs_all, _ = oracle.walk_pairs(walks, window)
    named_x = np.zeros(V, bool); named_x[pairs_all[:, 0]] = True
    named_c = np.zeros(V, bool); named_c[pairs_all[:, 1]] = True
    for row in negs.values():
        named_c[row] = True
    assert np.array_equal(Xg[~named_x].view(np.uint32), Xb[~named_x].view(np.uint32))
    assert np.array_equal(Cg[~named_c].view(np.uint32), Cb[~named_c].view(np.uint32))
    assert same_x[~named_x].all() and same_c[~named_c].all()


def test_walks_equal_pairs_when_sample_indices_agree():
    """window 1 on full walks: sample (r, i) has index r*L + i, which is what ne_train_batch uses for pair i of a
    call with sample_base r*L - the two GPU paths must then agree walk by walk."""
    V, d, K, n, L = 3000, 128, 5, 40, 10
    say("walks vs pairs on the GPU (window 1)")
    rng = np.random.default_rng(3)
    deg = (rng.pareto(1.0, V) * 3).astype(np.uint32) + 1
    walks = rng.integers(0, V, (n, L)).astype(np.int32)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at)
    tw, tp = make(V, d, n * L * 2, K, 5), make(V, d, n * L * 2, K, 5)
    ne.ne_train_walks(tw, alias, torch.from_numpy(walks).to(DEV), n, 1, K, [0.03], 0)       # all walks in one batch
    # the pair API numbers the samples of a call consecutively, so each walk is trained as a batch of its own
    tw2 = make(V, d, n * L * 2, K, 5)
    ne.ne_train_walks(tw2, alias, torch.from_numpy(walks).to(DEV), 1, 1, K, [0.03] * n, 0)
    for r in range(n):
        pairs = np.ascontiguousarray(np.stack([walks[r, :-1], walks[r, 1:]], axis=1).astype(np.int32))
        ne.ne_train_batch(tp, alias, torch.from_numpy(pairs).to(DEV), K, 0.03, r * L)
    torch.cuda.synchronize()
    ex = rowwise_rel_err(tw2.vertex.cpu().numpy(), tp.vertex.cpu().numpy())
    ec = rowwise_rel_err(tw2.context.cpu().numpy(), tp.context.cpu().numpy())
    say(f"  per-walk batches: walks vs pairs row error X {ex:.2e} C {ec:.2e}")
    assert ex <= 1e-5 and ec <= 1e-5
    # and batching matters: all walks in one batch is a different (still exact) step
    assert not torch.equal(tw.vertex, tw2.vertex)


def test_walks_argument_errors():
    V, d, K = 500, 64, 5
    t = make(V, d, 1000, K, 1)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(np.ones(V, np.uint32), 0, at)
    walks = torch.zeros((4, 10), dtype=torch.int32, device=DEV)
    before = t.vertex.clone()
    with pytest.raises(ne.NeError):
        ne.ne_train_walks(t, alias, walks, 4, 0, K, [0.1], 0)                 # window 0
    with pytest.raises(ne.NeError):
        ne.ne_train_walks(t, alias, walks, 4, 65, K, [0.1], 0)                # window too large
    with pytest.raises(ne.NeError):
        ne.ne_train_walks(t, alias, walks, 4, 5, K, [float("nan")], 0)        # lr not finite
    with pytest.raises(ne.NeError):
        ne.ne_train_walks(t, None, walks, 4, 5, K, [0.1], 0)                  # negatives without an alias table
    big = torch.zeros((400, 10), dtype=torch.int32, device=DEV)
    with pytest.raises(ne.NeError):
        ne.ne_train_walks(t, alias, big, 400, 5, K, [0.1], 0)                 # more references than the workspace holds
    ne.ne_train_walks(t, alias, walks[:0], 4, 5, K, [], 0)                    # no walks: no-op
    torch.cuda.synchronize()
    assert torch.equal(t.vertex, before)
