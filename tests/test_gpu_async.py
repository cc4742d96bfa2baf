"""Parity of the per-sample mode (ne_train_batch_async / ne_train_block_async).

Rows that one reference of a call names are updated exactly as in the minibatch step; rows that several
references name take every delta as atomic adds on the table row while other pairs may still be reading it.
No update is lost, but the result depends on timing wherever rows are shared, so there are three checks:
  * element by element on calls in which no row is named twice: equal to the oracle's minibatch step (and
    to the sequential one) to fp32 rounding;
  * negatives bit-exact always, and conservation on heavily shared rows: with scores pinned near zero
    (every coefficient is then +-1/2 whatever the timing) every row must receive the exact sum of its
    deltas - one lost update would show;
  * statistically: the loss curve against the sequential per-sample oracle at 256 and at 4096 pairs per
    call, each side evolving its own tables.  Inside a call the mode evaluates gradients at values between
    "before the call" and "fully updated", so its curve lies between the minibatch oracle's and the
    sequential oracle's; the bound is on the distance to the sequential one.
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


@pytest.mark.parametrize("block", [False, True])
def test_async_loses_no_update_on_shared_rows(block):
    """Every update must arrive, however many pairs of a call share a row.  All vertex rows hold the same vector
    e, the context table starts at zero and lr is tiny, so every score stays below 1e-5, every coefficient is
    1/2 (label 1) or -1/2 (label 0) to fp32 resolution, and context row r must end at
    (lr/2) (times named as context - times drawn as negative) e  whatever the timing.  One lost update would move
    the row by (lr/2) e; fp32 accumulation of at most 2500 terms stays below a tenth of that, so the bar is half
    an update, in absolute terms, on every row."""
    V, d, K, B, seed = 3000, 64, 5, 4096, 5
    say(f"async conservation on shared rows (block={block})")
    rng = np.random.default_rng(1)
    deg = (rng.pareto(1.0, V) * 3).astype(np.uint32) + 1
    e = np.linspace(0.01, 0.05, d).astype(np.float32)
    X0 = np.tile(e, (V, 1))
    C0 = np.zeros((V, d), np.float32)
    m = GpuModel(V, d, seed, deg, K, B, X=X0, C=C0)
    pairs = np.minimum((rng.pareto(0.8, (2 * B, 2)) * V / 50).astype(np.int64), rng.integers(0, V, (2 * B, 2))).astype(np.int32)
    pd = torch.from_numpy(pairs).cuda()
    lr = 1e-8
    neg_dev = torch.empty((2 * B, K), dtype=torch.int32, device="cuda:0")
    if block:
        ne.ne_train_block_async(m.tables, m.alias, pd, B, K, [lr, lr], 11, neg_dev)
    else:
        for i in range(2):
            ne.ne_train_batch_async(m.tables, m.alias, pd[i * B:(i + 1) * B], K, lr, 11 + i * B, neg_dev[i * B:(i + 1) * B])
    Xg, Cg = m.host_tables()
    thr, al, _ = oracle.build_alias(deg)
    neg = oracle.sample_negatives(seed, 11, 2 * B, K, thr, al)
    assert np.array_equal(neg_dev.cpu().numpy(), neg)
    as_ctx = np.bincount(pairs[:, 1], minlength=V)
    as_neg = np.bincount(neg.reshape(-1), minlength=V)
    named = as_ctx + as_neg
    say(f"  context rows are named up to {named.max()} times in the two calls; {(named > 1).sum()} rows more than once")
    assert 500 < named.max() < 2500
    want = 0.5 * np.float32(lr) * (as_ctx - as_neg).astype(np.float64)[:, None] * e.astype(np.float64)[None, :]
    update = 0.5 * lr * float(e.max())
    worst = np.abs(Cg.astype(np.float64) - want).max() / update
    say(f"  largest deviation from the exact sums: {worst:.3f} of one update")
    assert worst < 0.5
    assert np.array_equal(Xg, X0)                 # dx = lr * sum g_j c_j is far below fp32 resolution of x here


@pytest.mark.parametrize("B,nb,lr,every", [(256, 400, 0.2, 40), (4096, 100, 0.025, 10)])
def test_async_loss_curve_against_sequential_oracle(B, nb, lr, every):
    """256 pairs per call on R-MAT 20 k nodes, and config 1's shape (10 k nodes, 4096 pairs per call, lr 0.025):
    the loss on a fixed probe set, GPU per-sample mode against the sequential per-sample oracle, each side evolving
    its own tables.  Stated bound: within 4 % of the sequential oracle's loss at every probe, within 2.5 % at the end
    (measured 0.9 % / 0.4 % at 256 pairs per call and 2.7 % / 1.5 % at 4096: gradients inside a call are taken at
    values between those before the call and the fully updated ones, and the gap grows with the call)."""
    config1 = B == 4096
    V, d, K, seed = (10000 if config1 else 20000), 128, 5, 0
    say(f"async, loss curve vs sequential oracle ({B} pairs per call, {nb} calls)")
    g = wl.build_graph(V, wl.rmat_edges(V, 10 * V, seed=0))
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
        if t % every == 0 or t == nb - 1:
            m.loss.zero_()
            ne.ne_eval_loss(m.tables, m.alias, probe_d, K, 10**9, m.loss)
            lg = m.loss.item() / 4096
            ls = oracle.eval_loss(Xs, Cs, probe_n, probe_neg) / 4096
            worst = max(worst, abs(lg - ls) / ls)
            final_gap = abs(lg - ls) / ls
            first = first if first is not None else ls
            last = ls
            say(f"  call {t}: loss gpu per-sample {lg:.4f} sequential oracle {ls:.4f}")
        ne.ne_train_batch_async(m.tables, m.alias, pd, K, lr, s, m.neg_out)
        assert np.array_equal(m.neg_out[:B, :K].cpu().numpy(), neg_o)
        oracle.train_sequential(Xs, Cs, pn, neg_o, lr)
    say(f"  largest relative gap to the sequential oracle: {worst:.3%}, at the end {final_gap:.3%}")
    assert last < 0.97 * first          # the comparison is on a curve that actually moves
    assert worst <= 0.04 and final_gap <= 0.025
    Xg, Cg = m.host_tables()
    assert np.isfinite(Xg).all() and np.isfinite(Cg).all()


def test_async_needs_the_training_workspace():
    V, d = 200, 16
    vertex = torch.zeros((V, d), dtype=torch.float32, device="cuda:0")
    context = torch.zeros((V, d), dtype=torch.float32, device="cuda:0")
    t = ne.ne_create_tables(vertex, context, 0, init=False)          # evaluate-only handle
    pairs = torch.zeros((8, 2), dtype=torch.int32, device="cuda:0")
    with pytest.raises(ne.NeError):
        ne.ne_train_batch_async(t, None, pairs, 0, 0.1, 0)
    ne.ne_train_batch_async(t, None, pairs[:0], 0, 0.1, 0)            # empty batch: no-op
