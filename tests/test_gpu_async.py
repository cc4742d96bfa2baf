"""Parity of the unsynchronised per-sample mode (ne_train_batch_async).

Its result depends on timing wherever two pairs of a call name the same row, so there are two checks:
element by element on batches in which no row is named twice (there it must equal the oracle's
minibatch step, and the sequential one, to fp32 rounding), and statistically: negatives bit-exact, and a
loss curve that trails the sequential per-sample oracle by a bounded margin and closes in on it, each side
evolving its own tables (a row named by several pairs of one call keeps only one of their updates, so the
mode learns hub rows more slowly: parity for this mode is partial by construction).  With thousands of
pairs in flight on a small table that case is only required to stay finite and not to diverge.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2005_13789_amd as ne
import workloads as wl
from parity_util import GpuModel, rowwise_rel_err

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("V,d,K,B", [(60000, 128, 5, 512), (30000, 512, 10, 128), (9000, 64, 0, 3000), (20000, 100, 3, 300)])
def test_async_equals_oracle_without_collisions(V, d, K, B):
    say(f"async, collision-free V={V} d={d} K={K} B={B}")
    seed = 3
    rng = np.random.default_rng(d + K)
    X0 = rng.normal(0, 1.0 / np.sqrt(d), (V, d)).astype(np.float32)
    C0 = rng.normal(0, 1.0 / np.sqrt(d), (V, d)).astype(np.float32)
    deg = np.ones(V, np.uint32)                      # uniform negatives: collisions are rare and are removed below
    m = GpuModel(V, d, seed, deg if K > 0 else None, K, B, X=X0, C=C0)
    perm = rng.permutation(V).astype(np.int32)
    pairs = np.stack([perm[:B], perm[B:2 * B]], axis=1).copy()
    pd = torch.from_numpy(pairs).cuda()
    if K > 0:
        m.loss_sum(pd, 77)                           # learn the negatives, then drop every pair that collides
        neg = m.neg_out[:B, :K].cpu().numpy()
        ctx_all = np.concatenate([pairs[:, 1:2], neg], axis=1)
        u, cnt = np.unique(ctx_all, return_counts=True)
        dup = set(u[cnt > 1].tolist())
        keep = np.array([not (set(row.tolist()) & dup) for row in ctx_all])
        assert keep.sum() > B // 3
    else:
        neg = np.zeros((B, 0), np.int32)
        keep = np.ones(B, bool)
    # pairs that were dropped still advance the sample index: train the kept ones one call per run of kept pairs
    Xo, Co = X0.copy(), C0.copy()
    start = 0
    idx = np.flatnonzero(keep)
    runs = np.split(idx, np.flatnonzero(np.diff(idx) != 1) + 1)
    for run in runs:
        s, e = int(run[0]), int(run[-1]) + 1
        ne.ne_train_batch_async(m.tables, m.alias, pd[s:e], K, 0.05, 77 + s)
        oracle.train_batch(Xo, Co, np.ascontiguousarray(pairs[s:e]), np.ascontiguousarray(neg[s:e]), 0.05)
    Xg, Cg = m.host_tables()
    ex, ec = rowwise_rel_err(Xg, Xo), rowwise_rel_err(Cg, Co)
    say(f"  {int(keep.sum())} pairs in {len(runs)} calls: rowwise err X {ex:.2e} C {ec:.2e}")
    assert ex <= 1e-5 and ec <= 1e-5


def test_async_loss_curve_small_calls():
    """R-MAT 20 k nodes / 200 k edges, walks of 40, window 5, d=128, K=5, 400 calls of 256 pairs.  Even
    with 256 pairs in flight a hub row is named by several pairs of a call and keeps one of their
    updates, so the curve lags the sequential oracle (measured: up to 15 % mid-way, 4 % at the end) and
    closes in on it; the test bounds that lag."""
    say("async, loss curve vs sequential oracle (256 pairs per call)")
    V, d, K, B, seed, nb = 20000, 128, 5, 256, 0, 400
    g = wl.build_graph(V, wl.rmat_edges(V, 200000, seed=0))
    pairs_all = wl.walk_pairs(g, 40, 5, nb * B, seed=0)
    deg = g.degree.numpy().astype(np.uint32)
    m = GpuModel(V, d, seed, deg, K, B)
    Xs, Cs = oracle.init_tables(V, d, seed)
    thr, alias, _ = oracle.build_alias(deg)
    pd_all, pn_all = pairs_all.cuda(), pairs_all.numpy()
    probe_d, probe_n = pd_all[:4096], np.ascontiguousarray(pn_all[:4096])     # fixed evaluation set
    probe_neg = oracle.sample_negatives(seed, 10**9, 4096, K, thr, alias)
    worst, first, last, final_gap = 0.0, None, None, None
    for t in range(nb):
        s = t * B
        pd, pn = pd_all[s:s + B], np.ascontiguousarray(pn_all[s:s + B])
        neg_o = oracle.sample_negatives(seed, s, B, K, thr, alias)
        if t % 40 == 0 or t == nb - 1:
            m.loss.zero_()
            ne.ne_eval_loss(m.tables, m.alias, probe_d, K, 10**9, m.loss)
            lg = m.loss.item() / 4096
            ls = oracle.eval_loss(Xs, Cs, probe_n, probe_neg) / 4096
            worst = max(worst, abs(lg - ls) / ls)
            final_gap = abs(lg - ls) / ls
            first = first if first is not None else ls
            last = ls
            assert lg >= ls - 0.02 * ls       # never ahead of the lossless sequential run by more than noise
            say(f"  call {t}: loss gpu-async {lg:.4f} sequential {ls:.4f}")
        ne.ne_train_batch_async(m.tables, m.alias, pd, K, 0.2, s, m.neg_out)
        assert np.array_equal(m.neg_out[:B, :K].cpu().numpy(), neg_o)
        oracle.train_sequential(Xs, Cs, pn, neg_o, 0.2)
    say(f"  largest relative gap to the sequential oracle: {worst:.3%}")
    assert last < 0.97 * first          # the comparison is on a curve that actually moves
    assert worst <= 0.20 and final_gap <= 0.08


def test_async_under_contention_is_lossy_but_finite():
    """Config 1 with 4096 pairs in flight on a 10 k-row table: most rows are named by many pairs of a
    call and all but one of their updates are lost, so training is slower than the oracles; the mode
    must stay finite, keep the negatives exact and never increase the loss above its start."""
    say("async under contention (config 1, 4096 pairs per call)")
    V, d, K, B, seed, nb = 10000, 128, 5, 4096, 0, 30
    g = wl.build_graph(V, wl.rmat_edges(V, 100000, seed=0))
    pairs_all = wl.walk_pairs(g, 40, 5, nb * B, seed=0)
    deg = g.degree.numpy().astype(np.uint32)
    m = GpuModel(V, d, seed, deg, K, B)
    thr, alias, _ = oracle.build_alias(deg)
    pd_all = pairs_all.cuda()
    start = m.loss_sum(pd_all[:B], 0) / B
    for t in range(nb):
        s = t * B
        ne.ne_train_batch_async(m.tables, m.alias, pd_all[s:s + B], K, 0.025, s, m.neg_out)
        assert np.array_equal(m.neg_out[:B, :K].cpu().numpy(), oracle.sample_negatives(seed, s, B, K, thr, alias))
    end = m.loss_sum(pd_all[:B], 0) / B
    say(f"  loss {start:.4f} -> {end:.4f}")
    Xg, Cg = m.host_tables()
    assert np.isfinite(Xg).all() and np.isfinite(Cg).all() and end <= start + 1e-6
