"""Every setting of ne_set_tuning gives the oracle's result: rows that several references of a batch name
collect their deltas through per-reference buffer rows (the first list_cap references), through atomics
(the rest), or both, and the apply kernel sweeps 2, 4 or 8 positions per thread.  The inputs are hub-heavy so
that rows with 1, 2..list_cap and more than list_cap references all occur in one batch."""
import numpy as np
import pytest
import torch

import oracle
import paper_2005_13789_amd as ne
from parity_util import rowwise_rel_err
from test_gpu_walks import make, oracle_run

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

TUNINGS = [(0, 8), (0, 4), (0, 2), (1, 4), (3, 2), (8, 2), (8, 8), (-1, 0)]


def say(msg):
    print(msg, flush=True)


def hub_ids(rng, V, shape):
    """A third of the ids from 6 hubs, a third from a pool of V/20 (multiplicities of a few), the rest uniform."""
    n = int(np.prod(shape))
    kind = rng.integers(0, 3, n)
    ids = np.where(kind == 0, rng.integers(0, 6, n), np.where(kind == 1, rng.integers(6, 6 + max(V // 20, 1), n),
                                                             rng.integers(0, V, n)))
    return ids.astype(np.int32).reshape(shape)


@pytest.mark.parametrize("list_cap,sweep", TUNINGS)
@pytest.mark.parametrize("V,d,K,B,n_pairs", [(3000, 128, 5, 700, 1900), (900, 512, 10, 150, 400), (400, 36, 2, 300, 300)])
def test_pairs_with_tuning(V, d, K, B, n_pairs, list_cap, sweep):
    say(f"pairs V={V} d={d} K={K} B={B} n={n_pairs} list_cap={list_cap} sweep={sweep}")
    rng = np.random.default_rng(V + d + K)
    seed, base = 5, 77
    t = make(V, d, B, K, seed)
    ne.ne_set_tuning(t, list_cap, sweep)
    deg = (rng.pareto(1.0, V) * 3).astype(np.uint32) + 1
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at)
    thr, al, _ = oracle.build_alias(deg)
    pairs = hub_ids(rng, V, (n_pairs, 2))
    n_batches = -(-n_pairs // B)
    lrs = [0.02 / (1 + b) for b in range(n_batches)]
    Xo, Co = t.vertex.cpu().numpy(), t.context.cpu().numpy()
    Xb, Cb = Xo.copy(), Co.copy()
    neg_dev = torch.empty((n_pairs, K), dtype=torch.int32, device=DEV)
    ne.ne_train_block(t, alias, torch.from_numpy(pairs).to(DEV), B, K, lrs, base, neg_dev)
    torch.cuda.synchronize()
    neg = oracle.sample_negatives(seed, base, n_pairs, K, thr, al, 0)
    assert np.array_equal(neg_dev.cpu().numpy(), neg)
    for b in range(n_batches):
        oracle.train_batch(Xo, Co, pairs[b * B:(b + 1) * B], neg[b * B:(b + 1) * B], lrs[b])
    Xg, Cg = t.vertex.cpu().numpy(), t.context.cpu().numpy()
    ex, ec = rowwise_rel_err(Xg, Xo), rowwise_rel_err(Cg, Co)
    say(f"  row error X {ex:.2e} C {ec:.2e}")
    assert ex <= 1e-4 * n_batches and ec <= 1e-4 * n_batches
    named_x = np.zeros(V, bool); named_x[pairs[:, 0]] = True
    named_c = np.zeros(V, bool); named_c[pairs[:, 1]] = True; named_c[neg.reshape(-1)] = True
    assert np.array_equal(Xg[~named_x].view(np.uint32), Xb[~named_x].view(np.uint32))
    assert np.array_equal(Cg[~named_c].view(np.uint32), Cb[~named_c].view(np.uint32))
    # a second call on the same handle finds the hash state, the counters and the accumulators clean
    ne.ne_train_block(t, alias, torch.from_numpy(pairs[:B]).to(DEV), B, K, lrs[:1], base)
    torch.cuda.synchronize()
    oracle.train_batch(Xo, Co, pairs[:B], neg[:B], lrs[0])
    assert rowwise_rel_err(t.vertex.cpu().numpy(), Xo) <= 1e-4 * (n_batches + 1)
    assert rowwise_rel_err(t.context.cpu().numpy(), Co) <= 1e-4 * (n_batches + 1)


@pytest.mark.parametrize("list_cap,sweep", TUNINGS)
@pytest.mark.parametrize("V,d,K,n,L,window,wpb", [
    (600, 128, 5, 30, 20, 5, 12),     # one lane group per walk entry
    (600, 128, 5, 30, 48, 5, 12),     # by segments of a workgroup's entries
    (500, 256, 3, 12, 32, 4, 5),
])
def test_walks_with_tuning(V, d, K, n, L, window, wpb, list_cap, sweep):
    say(f"walks V={V} d={d} K={K} n={n} L={L} window={window} per batch={wpb} list_cap={list_cap} sweep={sweep}")
    rng = np.random.default_rng(V + n + L)
    seed, sample_base = 22, 500
    deg = (rng.pareto(1.0, V) * 3).astype(np.uint32) + 1
    walks = hub_ids(rng, V, (n, L))
    walks[0, L // 2:] = -1
    R = 1 + window * (K + 1)
    t = make(V, d, -(-(wpb * L * R) // (K + 2)), K, seed)
    ne.ne_set_tuning(t, list_cap, sweep)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at)
    thr, al, _ = oracle.build_alias(deg)
    n_batches = -(-n // wpb)
    lrs = [0.01 / (1 + b) for b in range(n_batches)]
    Xo, Co = t.vertex.cpu().numpy(), t.context.cpu().numpy()
    ne.ne_train_walks(t, alias, torch.from_numpy(walks).to(DEV), wpb, window, K, lrs, sample_base)
    torch.cuda.synchronize()
    oracle_run(Xo, Co, walks, wpb, window, K, lrs, seed, sample_base, thr, al)
    ex = rowwise_rel_err(t.vertex.cpu().numpy(), Xo)
    ec = rowwise_rel_err(t.context.cpu().numpy(), Co)
    say(f"  row error X {ex:.2e} C {ec:.2e}")
    assert ex <= 1e-4 * n_batches and ec <= 1e-4 * n_batches


def test_tuning_argument_errors():
    t = make(100, 8, 16, 2, 0)
    for bad in ((-2, 0), (9, 0), (0, 3), (0, 16), (0, -1)):
        with pytest.raises(ne.NeError):
            ne.ne_set_tuning(t, *bad)
    ne.ne_set_tuning(t, -1, 0)


@pytest.mark.parametrize("list_cap", [0, 1, 2, 7, 8])
@pytest.mark.parametrize("d", [128, 512])
def test_exact_multiplicities_around_the_list_capacity(list_cap, d):
    """Row k (k = 1..12) is named exactly k times as a source and row 100 + k exactly k times as a context, no
    negatives: lists shorter than, as long as and one short of the number of references, in one batch."""
    say(f"multiplicities 1..12, d={d}, list_cap={list_cap}")
    V, K = 400, 0
    src, ctx = [], []
    for k in range(1, 13):
        for i in range(k):
            src.append(k); ctx.append(200 + 13 * k + i)          # source row k, k times, with distinct contexts
            src.append(300 + (7 * k + i) % 90); ctx.append(100 + k)   # context row 100 + k, k times
    rng = np.random.default_rng(d + list_cap)
    order = rng.permutation(len(src))
    pairs = np.stack([np.array(src)[order], np.array(ctx)[order]], axis=1).astype(np.int32)
    B = pairs.shape[0]
    t = make(V, d, B, K, 3)
    ne.ne_set_tuning(t, list_cap, 0)
    Xo, Co = t.vertex.cpu().numpy(), t.context.cpu().numpy()
    for rep in range(2):       # the second batch finds counters, lists and accumulators clean
        ne.ne_train_batch(t, None, torch.from_numpy(pairs).to(DEV), K, 0.05, 0)
        torch.cuda.synchronize()
        oracle.train_batch(Xo, Co, pairs, np.zeros((B, 0), np.int32), 0.05)
        ex = rowwise_rel_err(t.vertex.cpu().numpy(), Xo)
        ec = rowwise_rel_err(t.context.cpu().numpy(), Co)
        say(f"  batch {rep}: row error X {ex:.2e} C {ec:.2e}")
        assert ex <= 1e-5 * (rep + 1) and ec <= 1e-5 * (rep + 1)
