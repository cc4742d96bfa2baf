"""GPU-vs-oracle parity through the C ABI (run with -m gpu on an MI355X).

Bars: bit-exact for table initialisation, alias tables and negative ids; row-wise max relative error
of the updated fp32 tables <= 1e-4 after one batch and <= 1e-3 after 100 batches; per-batch loss within
1 %; rows a batch does not name stay bit-identical.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2005_13789_amd as ne
import workloads as wl
from parity_util import GpuModel, oracle_negatives, rowwise_rel_err, table_rel_err

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("V,d,seed", [(3001, 128, 0), (257, 100, 1), (64, 512, 2**40 + 3), (5, 4, 9), (33, 1024, 4)])
def test_init_bit_exact(V, d, seed):
    say(f"init V={V} d={d} seed={seed}")
    m = GpuModel(V, d, seed, None, 0, 1)
    X, C = m.host_tables()
    Xo, Co = oracle.init_tables(V, d, seed)
    assert np.array_equal(X.view(np.uint32), Xo.view(np.uint32))
    assert np.array_equal(C.view(np.uint32), Co.view(np.uint32))


@pytest.mark.parametrize("n,base,seed", [(1, 0, 0), (2, 5, 1), (1000, 0, 2), (65537, 1000, 3)])
def test_alias_table_bit_exact(n, base, seed):
    say(f"alias n={n} base={base}")
    rng = np.random.default_rng(seed)
    deg = (rng.pareto(1.1, n) * 3).astype(np.uint32)
    deg[rng.integers(0, n)] += 2
    thr, alias, _ = oracle.build_alias(deg)
    table = torch.empty((n, 2), dtype=torch.int32, device="cuda:0")
    h = ne.ne_build_neg_alias(deg, base, table)
    got = table.cpu().numpy().view(np.uint32)
    assert np.array_equal(got[:, 0], thr) and np.array_equal(got[:, 1], alias)
    assert h.n == n and h.base == base


@pytest.mark.parametrize("d,K,B,sample_base", [(128, 5, 4096, 0), (128, 5, 1000, 2**32 - 300), (64, 10, 777, 2**40),
                                               (512, 10, 300, 12345), (8, 1, 5, 0), (256, 62, 130, 7), (100, 15, 513, 1)])
def test_negative_ids_bit_exact(d, K, B, sample_base):
    say(f"negatives d={d} K={K} B={B} base={sample_base}")
    V, seed = 5000, 0xABCDEF0123
    rng = np.random.default_rng(K)
    deg = (rng.pareto(1.0, V) * 2).astype(np.uint32) + (rng.random(V) < 0.7)
    m = GpuModel(V, d, seed, deg, K, B)
    pairs = torch.from_numpy(rng.integers(0, V, (B, 2)).astype(np.int32)).cuda()
    m.loss_sum(pairs, sample_base)
    got = m.neg_out[:B, :K].cpu().numpy()
    want = oracle_negatives(seed, sample_base, B, K, deg)
    assert np.array_equal(got, want)


def run_case(V, d, K, B, n_batches, seed, lr0=0.025, scale=None, base=0, n_alias=None, tol=1e-4):
    """Train n_batches on random pairs from both sides; returns the per-batch records."""
    rng = np.random.default_rng(seed + 17)
    n_alias = V if n_alias is None else n_alias
    deg = (rng.pareto(1.0, n_alias) * 2).astype(np.uint32) + (rng.random(n_alias) < 0.7)
    deg[0] += 1
    # skewed ids so that rows repeat inside a batch (hubs), as on an R-MAT graph
    def ids(n):
        return np.minimum((rng.pareto(0.8, n) * V / 50).astype(np.int64), rng.integers(0, V, n)).astype(np.int32)
    Xo, Co = oracle.init_tables(V, d, seed)
    if scale is not None:                # start from non-trivial tables so that scores are not all zero
        Xo = (rng.normal(0, scale, (V, d))).astype(np.float32)
        Co = (rng.normal(0, scale, (V, d))).astype(np.float32)
        m = GpuModel(V, d, seed, deg, K, B, base=base, X=Xo, C=Co)
    else:
        m = GpuModel(V, d, seed, deg, K, B, base=base)
    thr, alias, _ = oracle.build_alias(deg) if K > 0 else (None, None, None)
    sample_base = 0
    for t in range(n_batches):
        nb = B if t % 3 != 2 else max(1, B - 37)          # ragged batches in between
        pairs = np.stack([ids(nb), ids(nb)], axis=1).astype(np.int32)
        pd = torch.from_numpy(pairs).cuda()
        lr = wl.linear_decay_lr(lr0, sample_base, n_batches * B)
        neg_o = oracle.sample_negatives(seed, sample_base, nb, K, thr, alias, base) if K > 0 else np.zeros((nb, 0), np.int32)
        loss_g = m.loss_sum(pd, sample_base)
        loss_o = oracle.eval_loss(Xo, Co, pairs, neg_o)
        # one evaluation at identical tables (batch 0) is fp32 terms against fp64: 1e-5; later batches compare
        # two trajectories (each side evolves its own tables), where the bar is the loss curve's 1 %
        assert abs(loss_g - loss_o) <= (1e-5 if t == 0 else 0.01) * abs(loss_o), (t, loss_g, loss_o)
        Xb, Cb = (m.host_tables() if t == 0 else (None, None))
        neg_g = m.train(pd, lr, sample_base)
        assert np.array_equal(neg_g, neg_o), f"negative ids differ in batch {t}"
        oracle.train_batch(Xo, Co, pairs, neg_o, lr)
        if t == 0:
            Xg, Cg = m.host_tables()
            ex, ec = rowwise_rel_err(Xg, Xo), rowwise_rel_err(Cg, Co)
            say(f"  batch 0: rowwise err X {ex:.2e} C {ec:.2e}")
            assert ex <= tol and ec <= tol
            touchedX = np.zeros(V, bool); touchedX[pairs[:, 0]] = True
            touchedC = np.zeros(V, bool); touchedC[pairs[:, 1]] = True; touchedC[neg_o.reshape(-1)] = True
            assert np.array_equal(Xg[~touchedX].view(np.uint32), Xb[~touchedX].view(np.uint32))
            assert np.array_equal(Cg[~touchedC].view(np.uint32), Cb[~touchedC].view(np.uint32))
        sample_base += nb
    Xg, Cg = m.host_tables()
    return Xg, Cg, Xo, Co


def test_first_batch_from_init_config1_shape():
    """Config-1 shape: V=10k, d=128, K=5, B=4096 from the U(+-0.5/d) / zero init.  C = 0 means dx = 0:
    the vertex table must stay bit-identical and context must match to 1e-4 row-wise."""
    say("first batch, config-1 shape")
    V, d, K, B, seed = 10000, 128, 5, 4096, 0
    X0, _ = oracle.init_tables(V, d, seed)
    Xg, Cg, Xo, Co = run_case(V, d, K, B, 1, seed)
    assert np.array_equal(Xg.view(np.uint32), X0.view(np.uint32))
    assert rowwise_rel_err(Cg, Co) <= 1e-4


@pytest.mark.parametrize("V,d,K,B", [(2000, 128, 5, 1000), (500, 4, 0, 64), (500, 8, 1, 1), (800, 64, 7, 257),
                                     (3000, 96, 5, 1500), (3000, 100, 5, 999), (1500, 256, 10, 640),
                                     (1200, 512, 10, 300), (700, 1024, 15, 130), (900, 128, 31, 200),
                                     (900, 32, 62, 100), (4000, 128, 5, 3)])
def test_one_batch_shapes(V, d, K, B):
    say(f"one batch V={V} d={d} K={K} B={B}")
    run_case(V, d, K, B, 1, seed=d * 1000 + K, scale=0.5 / math.sqrt(d) * 3)


def test_alias_block_with_base():
    """Negatives restricted to a context block [base, base+n) (a GPU's fixed context partition)."""
    say("block-local negatives")
    V, d, K, B = 4000, 128, 5, 2048
    Xg, Cg, Xo, Co = run_case(V, d, K, B, 2, seed=5, scale=0.2, base=1000, n_alias=1000)
    assert rowwise_rel_err(Cg, Co) <= 1e-3


def test_config1_100_batches():
    """Config 1 end to end: R-MAT 10k nodes / 100k edges, walks of 40, window 5, d=128, K=5, B=4096,
    lr 0.025 with linear decay, seed 0; first 100 batches."""
    say("config 1, 100 batches")
    V, d, K, B, seed, nb = 10000, 128, 5, 4096, 0, 100
    g = wl.build_graph(V, wl.rmat_edges(V, 100000, seed=0))
    pairs_all = wl.walk_pairs(g, 40, 5, 1_000_000, seed=0)
    deg = g.degree.numpy().astype(np.uint32)
    total = pairs_all.shape[0]
    m = GpuModel(V, d, seed, deg, K, B)
    Xo, Co = oracle.init_tables(V, d, seed)
    thr, alias, _ = oracle.build_alias(deg)
    pairs_dev = pairs_all.cuda()
    pairs_np = pairs_all.numpy()
    losses = []
    for t in range(nb):
        s = t * B
        pd, pn = pairs_dev[s:s + B], pairs_np[s:s + B]
        lr = wl.linear_decay_lr(0.025, s, total)
        neg_o = oracle.sample_negatives(seed, s, B, K, thr, alias)
        lg, lo = m.loss_sum(pd, s) / B, oracle.eval_loss(Xo, Co, pn, neg_o) / B
        losses.append((lg, lo))
        assert abs(lg - lo) <= 0.01 * lo, (t, lg, lo)
        neg_g = m.train(pd, lr, s)
        assert np.array_equal(neg_g, neg_o), t
        oracle.train_batch(Xo, Co, pn, neg_o, lr)
        if t == 0:
            Xg, Cg = m.host_tables()
            assert rowwise_rel_err(Xg, Xo) <= 1e-4 and rowwise_rel_err(Cg, Co) <= 1e-4
            assert abs(lo - 6 * math.log(2)) < 1e-12
    Xg, Cg = m.host_tables()
    ex, ec = rowwise_rel_err(Xg, Xo), rowwise_rel_err(Cg, Co)
    say(f"  after {nb} batches: rowwise err X {ex:.2e} C {ec:.2e}; loss {losses[0][0]:.4f} -> {losses[-1][0]:.4f}")
    assert ex <= 1e-3 and ec <= 1e-3
    assert table_rel_err(Xg, Xo) <= 1e-3 and table_rel_err(Cg, Co) <= 1e-3
    assert losses[-1][0] < losses[0][0]


@pytest.mark.parametrize("V,d,K,B,scale", [(5000, 128, 5, 4096, 0.3), (3000, 512, 10, 700, 0.1), (800, 64, 0, 333, 0.5),
                                           (2000, 256, 31, 257, 0.2), (4000, 100, 5, 1, 1.0), (6000, 128, 5, 65536, 0.4)])
def test_eval_loss_single_call_precision(V, d, K, B, scale):
    """ne_eval_loss at tables identical to the oracle's: fp32 dot products and softplus terms, fp64 sum,
    against fp64 throughout.  A term's error is ~d * 2^-24 of its score plus one ulp of the term and the
    errors of the B(K+1) terms do not line up, so one call sits near 1e-7; the bar is 1e-5.  Scores reach
    several units here (large |score| exercises both branches of the stable softplus)."""
    say(f"eval_loss precision V={V} d={d} K={K} B={B}")
    rng = np.random.default_rng(V + d)
    deg = (rng.pareto(1.0, V) * 2).astype(np.uint32) + 1
    X = rng.normal(0, scale, (V, d)).astype(np.float32)
    C = rng.normal(0, scale, (V, d)).astype(np.float32)
    m = GpuModel(V, d, 3, deg, K, B, X=X, C=C)
    pairs = rng.integers(0, V, (B, 2)).astype(np.int32)
    neg_o = oracle_negatives(3, 99, B, K, deg)
    lg = m.loss_sum(torch.from_numpy(pairs).cuda(), 99)
    lo = oracle.eval_loss(X, C, pairs, neg_o)
    say(f"  loss/pair {lo / B:.4f}, relative difference {abs(lg - lo) / lo:.2e}")
    assert abs(lg - lo) <= 1e-5 * lo


def test_empty_batch_and_validate():
    say("empty batch, validate")
    V, d, K = 100, 16, 3
    m = GpuModel(V, d, 1, np.ones(V, np.uint32), K, 8)
    X0, C0 = m.host_tables()
    empty = torch.empty((0, 2), dtype=torch.int32, device="cuda:0")
    m.train(empty, 0.1, 0, want_neg=False)
    X1, C1 = m.host_tables()
    assert np.array_equal(X0, X1) and np.array_equal(C0, C1)
    bad = torch.zeros((), dtype=torch.int64, device="cuda:0")
    pairs = torch.tensor([[0, 99], [100, 5], [-1, 3], [7, 7]], dtype=torch.int32, device="cuda:0")
    ne.ne_validate_pairs(m.tables, pairs, bad)
    assert int(bad.item()) == 2
    with pytest.raises(ne.NeError):          # batch larger than the workspace was sized for
        ne.ne_train_batch(m.tables, m.alias, pairs.repeat(3, 1), K, 0.1, 0)
    with pytest.raises(ne.NeError):          # more negatives than the workspace was sized for
        ne.ne_train_batch(m.tables, m.alias, pairs[:1], K + 1, 0.1, 0)
    # alias range outside the tables
    with pytest.raises(ne.NeError):
        t2 = torch.empty((200, 2), dtype=torch.int32, device="cuda:0")
        a2 = ne.ne_build_neg_alias(np.ones(200, np.uint32), 0, t2)
        ne.ne_train_batch(m.tables, a2, pairs[:1], K, 0.1, 0)


def test_train_block_matches_oracle_and_single_batches():
    """ne_train_block (claim/resolve of batch i+1 fused into the kernels of batch i) on a run of
    batches with a ragged tail: equals the oracle, and equals ne_train_batch called per batch."""
    say("train_block")
    V, d, K, B, seed = 6000, 128, 5, 2048, 3
    n_pairs = 11 * B + 777
    nb = -(-n_pairs // B)
    rng = np.random.default_rng(1)
    deg = (rng.pareto(1.0, V) * 2).astype(np.uint32) + 1
    X0 = rng.normal(0, 0.2, (V, d)).astype(np.float32)
    C0 = rng.normal(0, 0.2, (V, d)).astype(np.float32)
    ids = np.minimum((rng.pareto(0.8, (n_pairs, 2)) * V / 50).astype(np.int64), V - 1).astype(np.int32)
    lrs = [wl.linear_decay_lr(0.05, i * B, n_pairs) for i in range(nb)]
    pairs_dev = torch.from_numpy(ids).cuda()
    base = 2**33 + 11

    m = GpuModel(V, d, seed, deg, K, B, X=X0, C=C0)
    negs = torch.empty((n_pairs, K), dtype=torch.int32, device="cuda:0")
    ne.ne_train_block(m.tables, m.alias, pairs_dev, B, K, lrs, base, negs)
    Xg, Cg = m.host_tables()

    thr, alias, _ = oracle.build_alias(deg)
    Xo, Co = X0.copy(), C0.copy()
    neg_all = oracle.sample_negatives(seed, base, n_pairs, K, thr, alias)
    assert np.array_equal(negs.cpu().numpy(), neg_all)
    for i in range(nb):
        sl = slice(i * B, min((i + 1) * B, n_pairs))
        oracle.train_batch(Xo, Co, np.ascontiguousarray(ids[sl]), np.ascontiguousarray(neg_all[sl]), lrs[i])
    ex, ec = rowwise_rel_err(Xg, Xo), rowwise_rel_err(Cg, Co)
    say(f"  block vs oracle: rowwise err X {ex:.2e} C {ec:.2e}")
    assert ex <= 1e-3 and ec <= 1e-3

    m2 = GpuModel(V, d, seed, deg, K, B, X=X0, C=C0)
    for i in range(nb):
        sl = slice(i * B, min((i + 1) * B, n_pairs))
        ne.ne_train_batch(m2.tables, m2.alias, pairs_dev[sl], K, lrs[i], base + i * B)
    X2, C2 = m2.host_tables()
    assert rowwise_rel_err(Xg, X2) <= 1e-4 and rowwise_rel_err(Cg, C2) <= 1e-4
    # a second block on the same handle starts from clean hash state
    ne.ne_train_block(m.tables, m.alias, pairs_dev[:3 * B + 5], B, K, lrs[:4], 0)
    for i in range(4):
        sl = slice(i * B, min((i + 1) * B, 3 * B + 5))
        neg_o = oracle.sample_negatives(seed, i * B, sl.stop - sl.start, K, thr, alias)
        oracle.train_batch(Xo, Co, np.ascontiguousarray(ids[sl]), neg_o, lrs[i])
    Xg, Cg = m.host_tables()
    assert rowwise_rel_err(Xg, Xo) <= 1e-3 and rowwise_rel_err(Cg, Co) <= 1e-3


@pytest.mark.parametrize("V,d,K,B,n_pairs", [(3000, 512, 10, 512, 5 * 512 + 100), (2500, 64, 0, 1024, 4 * 1024), (800, 128, 62, 64, 5 * 64 + 1),
                                             (50, 128, 5, 2048, 6 * 2048)])
def test_train_block_shapes(V, d, K, B, n_pairs):
    """ne_train_block over other lane-group shapes, K = 0, the largest K, and a table so small that
    almost every row is named many times per batch (the shared-row path carries nearly everything)."""
    say(f"train_block V={V} d={d} K={K} B={B} n_pairs={n_pairs}")
    seed = 21
    rng = np.random.default_rng(V + d)
    deg = (rng.pareto(1.0, V) * 2).astype(np.uint32) + 1
    X0 = rng.normal(0, 1.0 / np.sqrt(d), (V, d)).astype(np.float32)
    C0 = rng.normal(0, 1.0 / np.sqrt(d), (V, d)).astype(np.float32)
    ids = rng.integers(0, V, (n_pairs, 2)).astype(np.int32)
    nb = -(-n_pairs // B)
    lrs = [0.02] * nb
    m = GpuModel(V, d, seed, deg if K > 0 else None, K, B, X=X0, C=C0)
    ne.ne_train_block(m.tables, m.alias, torch.from_numpy(ids).cuda(), B, K, lrs, 5)
    Xg, Cg = m.host_tables()
    Xo, Co = X0.copy(), C0.copy()
    if K > 0:
        thr, alias, _ = oracle.build_alias(deg)
    for i in range(nb):
        sl = slice(i * B, min((i + 1) * B, n_pairs))
        neg_o = (oracle.sample_negatives(seed, 5 + i * B, sl.stop - sl.start, K, thr, alias) if K > 0
                 else np.zeros((sl.stop - sl.start, 0), np.int32))
        oracle.train_batch(Xo, Co, np.ascontiguousarray(ids[sl]), neg_o, lrs[i])
    ex, ec = rowwise_rel_err(Xg, Xo), rowwise_rel_err(Cg, Co)
    say(f"  rowwise err X {ex:.2e} C {ec:.2e}")
    assert ex <= 1e-3 and ec <= 1e-3


def test_long_run_keeps_hash_state_clean():
    """400 batches on one handle, alternating ne_train_block runs of different lengths and batch sizes
    with single ne_train_batch calls: any stale hash position or slot would show up as drift."""
    say("long run, 400 batches")
    V, d, K, seed = 4000, 64, 5, 9
    rng = np.random.default_rng(5)
    deg = (rng.pareto(1.0, V) * 2).astype(np.uint32) + 1
    X0 = rng.normal(0, 0.1, (V, d)).astype(np.float32)
    C0 = rng.normal(0, 0.1, (V, d)).astype(np.float32)
    m = GpuModel(V, d, seed, deg, K, 1024, X=X0, C=C0)
    thr, alias, _ = oracle.build_alias(deg)
    Xo, Co = X0.copy(), C0.copy()
    done, base = 0, 0
    while done < 400:
        B = int(rng.choice([1024, 512, 333]))
        nb = int(rng.integers(1, 9))
        n_pairs = nb * B - int(rng.integers(0, B // 2))
        ids = np.minimum((rng.pareto(0.9, (n_pairs, 2)) * V / 40).astype(np.int64), V - 1).astype(np.int32)
        pd = torch.from_numpy(ids).cuda()
        if nb == 1:
            ne.ne_train_batch(m.tables, m.alias, pd, K, 0.01, base)
        else:
            ne.ne_train_block(m.tables, m.alias, pd, B, K, [0.01] * nb, base)
        for i in range(-(-n_pairs // B) if nb > 1 else 1):
            sl = slice(i * B, min((i + 1) * B, n_pairs)) if nb > 1 else slice(0, n_pairs)
            neg_o = oracle.sample_negatives(seed, base + sl.start, sl.stop - sl.start, K, thr, alias)
            oracle.train_batch(Xo, Co, np.ascontiguousarray(ids[sl]), neg_o, 0.01)
        base += n_pairs
        done += nb
    Xg, Cg = m.host_tables()
    ex, ec = rowwise_rel_err(Xg, Xo), rowwise_rel_err(Cg, Co)
    say(f"  after {done} batches: rowwise err X {ex:.2e} C {ec:.2e}")
    assert ex <= 2e-3 and ec <= 2e-3
