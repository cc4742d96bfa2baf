"""Parity at the benchmark's full sizes and launch configuration (ne_train_runs / ne_train_block, batch 65536).

Config 2 (1 M nodes): the oracle runs the same batches on host copies of the tables; every element is
compared.  Config 3 (100 M nodes, 102 GB of tables): host copies are impossible, so sampled table rows
are checked one by one: for a sample of touched rows, every pair of the batch that names one of them
is collected, the pre-batch values of all rows those pairs read are fetched, and the oracle runs on
that sub-batch (ids renumbered); its result for the sampled rows is exact because a row's update
depends only on the pairs that name it.  Plus properties that hold at any size: negatives bit-exact and
inside the context block, rows no pair names bit-identical.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2005_13789_amd as ne
import workloads as wl
from parity_util import rowwise_rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def make_tables(V, d, K, B, seed):
    vertex = torch.empty((V, d), dtype=torch.float32, device=DEV)
    context = torch.empty((V, d), dtype=torch.float32, device=DEV)
    ws = torch.empty(ne.ne_workspace_bytes(d, B, K), dtype=torch.uint8, device=DEV)
    t = ne.ne_create_tables(vertex, context, seed, init=True, max_batch=B, max_negatives=K, workspace=ws)
    return t


def test_config2_full_compare():
    say("config 2: 1M nodes, 20M edges, walks of 80, window 5, B=65536; 3 batches, every element")
    V, d, K, B, seed, nb = 1_000_000, 128, 5, 65536, 1, 3
    g = wl.build_graph(V, wl.rmat_edges(V, 20_000_000, seed, device=DEV))
    pairs = wl.walk_pairs(g, 80, 5, nb * B, seed)
    deg = g.degree.cpu().numpy().astype(np.uint32)
    del g
    t = make_tables(V, d, K, B, seed)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at)
    # two warm-up batches so that the compared batches start from non-trivial tables
    lrs = [0.025, 0.02, 0.015]
    neg = torch.empty((nb * B, K), dtype=torch.int32, device=DEV)
    X0 = None
    ne.ne_train_block(t, alias, pairs[:B], B, K, lrs[:1], 0, neg[:B])
    torch.cuda.synchronize()
    Xo, Co = t.vertex.cpu().numpy(), t.context.cpu().numpy()
    ne.ne_train_block(t, alias, pairs[B:], B, K, lrs[1:], B, neg[B:])
    torch.cuda.synchronize()
    thr, al, _ = oracle.build_alias(deg)
    pn = pairs.cpu().numpy()
    neg_all = oracle.sample_negatives(seed, 0, nb * B, K, thr, al)
    assert np.array_equal(neg.cpu().numpy(), neg_all)
    Xpre, Cpre = Xo.copy(), Co.copy()
    for i in (1, 2):
        sl = slice(i * B, (i + 1) * B)
        oracle.train_batch(Xo, Co, np.ascontiguousarray(pn[sl]), np.ascontiguousarray(neg_all[sl]), lrs[i])
    Xg, Cg = t.vertex.cpu().numpy(), t.context.cpu().numpy()
    ex, ec = rowwise_rel_err(Xg, Xo), rowwise_rel_err(Cg, Co)
    say(f"  rowwise err X {ex:.2e} C {ec:.2e}")
    assert ex <= 1e-4 and ec <= 1e-4       # two batches from a common starting point
    touched_x = np.zeros(V, bool); touched_x[pn[B:, 0]] = True
    touched_c = np.zeros(V, bool); touched_c[pn[B:, 1]] = True; touched_c[neg_all[B:].reshape(-1)] = True
    assert np.array_equal(Xg[~touched_x].view(np.uint32), Xpre[~touched_x].view(np.uint32))
    assert np.array_equal(Cg[~touched_c].view(np.uint32), Cpre[~touched_c].view(np.uint32))


def sampled_row_check(t, alias, pairs_dev, K, lr, sample_base, n_sample, rng):
    """Train one batch with ne_train_block and check n_sample touched rows of each table."""
    B = pairs_dev.shape[0]
    d = t.dim
    neg = torch.empty((B, K), dtype=torch.int32, device=DEV)
    loss = torch.zeros((), dtype=torch.float64, device=DEV)
    ne.ne_eval_loss(t, alias, pairs_dev, K, sample_base, loss, neg)      # same draws as training
    torch.cuda.synchronize()
    p = pairs_dev.long()
    cref = torch.cat([p[:, 1:2], neg.long()], dim=1)                     # [B][K+1] context rows per pair
    # sample: a mix of rows named once and rows named often
    cu, cc = torch.unique(cref.reshape(-1), return_counts=True)
    xu, xc = torch.unique(p[:, 0], return_counts=True)
    def pick(u, c):
        hot = u[torch.argsort(c, descending=True)[: n_sample // 4]]
        rest = u[torch.from_numpy(rng.choice(u.numel(), n_sample - hot.numel(), replace=False)).to(DEV)]
        return torch.unique(torch.cat([hot, rest]))
    srows_c, srows_x = pick(cu, cc), pick(xu, xc)
    sel = torch.isin(p[:, 0], srows_x) | torch.isin(cref, srows_c).any(dim=1)
    sub_pairs, sub_neg = p[sel], neg.long()[sel]
    say(f"  {int(sel.sum())} pairs name one of {srows_x.numel()} + {srows_c.numel()} sampled rows")
    # renumber the rows the sub-batch reads and fetch their pre-batch values
    xs, xinv = torch.unique(sub_pairs[:, 0], return_inverse=True)
    cs, cinv = torch.unique(torch.cat([sub_pairs[:, 1:2], sub_neg], dim=1), return_inverse=True)
    n = max(xs.numel(), cs.numel())
    Xm = np.zeros((n, d), np.float32); Cm = np.zeros((n, d), np.float32)
    Xm[: xs.numel()] = t.vertex[xs].cpu().numpy()
    Cm[: cs.numel()] = t.context[cs].cpu().numpy()
    mp = np.stack([xinv.cpu().numpy(), cinv[:, 0].cpu().numpy()], axis=1).astype(np.int32)
    mn = np.ascontiguousarray(cinv[:, 1:].cpu().numpy().astype(np.int32))
    # untouched sample for the bit-identical check
    probe = torch.from_numpy(rng.integers(0, t.num_nodes, 4096)).to(DEV)
    probe_c = probe[~torch.isin(probe, cu)]
    probe_x = probe[~torch.isin(probe, xu)]
    before_c, before_x = t.context[probe_c].clone(), t.vertex[probe_x].clone()

    negs_train = torch.empty_like(neg)
    ne.ne_train_block(t, alias, pairs_dev, B, K, [lr], sample_base, negs_train)
    torch.cuda.synchronize()
    assert torch.equal(negs_train, neg)
    oracle.train_batch(Xm, Cm, mp, mn, lr)
    gx = t.vertex[srows_x].cpu().numpy()
    gc = t.context[srows_c].cpu().numpy()
    ox = Xm[torch.searchsorted(xs, srows_x).cpu().numpy()]
    oc = Cm[torch.searchsorted(cs, srows_c).cpu().numpy()]
    ex, ec = rowwise_rel_err(gx, ox), rowwise_rel_err(gc, oc)
    say(f"  sampled rows: rowwise err X {ex:.2e} C {ec:.2e}")
    assert ex <= 1e-4 and ec <= 1e-4
    assert torch.equal(t.context[probe_c], before_c) and torch.equal(t.vertex[probe_x], before_x)
    return neg


def test_config3_sampled_rows():
    say("config 3: 100M nodes, d=128, K=5, B=65536, 4x4 buckets, negatives inside the context block")
    V, d, K, B, seed, grid = 100_000_000, 128, 5, 65536, 2, 4
    rng = np.random.default_rng(0)
    degree = wl.rmat_degrees(V, 400_000_000, seed, device=DEV)          # a fifth of the edges: same shape, less set-up
    pairs = wl.rmat_pairs(V, 80 * B, seed, device=DEV)
    bp = wl.bucket_pairs(pairs, V, grid)
    sched = [s for s in wl.orthogonal_schedule(bp, B) if s[1] == B]
    t = make_tables(V, d, K, B, seed)
    s0, n0, bi, bj = sched[0]
    lo, hi = bj * bp.block_rows, min((bj + 1) * bp.block_rows, V)
    deg_blk = degree[lo:hi].clamp(max=2**32 - 1).cpu().numpy().astype(np.uint32)
    at = torch.empty((hi - lo, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg_blk, lo, at)
    # batches of the same bucket: the first from the initial tables, the later ones from trained tables
    same = [s for s in sched if (s[2], s[3]) == (bi, bj)][:3]
    assert len(same) >= 2
    thr, al, _ = oracle.build_alias(deg_blk)
    for k, (s, n, _, _) in enumerate(same):
        if k == 2:       # the last batch through the per-reference lists, which are off by default at this size
            ne.ne_set_tuning(t, 8, 2)
        pd = bp.pairs[s:s + n]
        assert int((pd[:, 0].long() // bp.block_rows != bi).sum()) == 0
        neg = sampled_row_check(t, alias, pd, K, 0.025, 1000 * k, 256, rng)
        assert int(neg.min()) >= lo and int(neg.max()) < hi
        want = oracle.sample_negatives(seed, 1000 * k, 2048, K, thr, al, lo)
        assert np.array_equal(neg[:2048].cpu().numpy(), want)


def test_config3_runs_in_the_benchmark_configuration():
    """bench.py trains config 3 through ne_train_runs: the runs of consecutive batches of the (src-block, ctx-block)
    buckets in one call, every batch's id-only work riding in the launches of the batch before it, also across a
    change of bucket and alias table.  Here: two buckets of the orthogonal order, three batches each, in that
    configuration; then, from the same initial tables (the seeded init is reproducible), the same batches one call
    each, every one checked against the oracle on sampled rows; the two end states must agree on every row the
    batches name (sampled) to 1e-5 - the arithmetic is the same, only the order of atomic adds differs - and
    bit for bit on rows they do not name."""
    say("config 3 through ne_train_runs: 2 buckets x 3 batches of 65536, 100M nodes")
    V, d, K, B, seed, grid = 100_000_000, 128, 5, 65536, 2, 4
    rng = np.random.default_rng(3)
    degree = wl.rmat_degrees(V, 400_000_000, seed, device=DEV)
    pairs = wl.rmat_pairs(V, 100 * B, seed, device=DEV)
    bp = wl.bucket_pairs(pairs, V, grid)
    sched = [s for s in wl.orthogonal_schedule(bp, B) if s[1] == B]
    buckets = []
    for s in sched:                                   # the first two buckets of the schedule with three whole batches
        key = (s[2], s[3])
        if key not in [b[0] for b in buckets]:
            same = [x for x in sched if (x[2], x[3]) == key][:3]
            if len(same) == 3 and same[2][0] == same[0][0] + 2 * B:
                buckets.append((key, same))
        if len(buckets) == 2:
            break
    assert len(buckets) == 2 and buckets[0][0][0] != buckets[1][0][0] and buckets[0][0][1] != buckets[1][0][1]
    aliases, oracles = {}, {}
    for (bi, bj), _ in buckets:
        lo, hi = bj * bp.block_rows, min((bj + 1) * bp.block_rows, V)
        deg_blk = degree[lo:hi].clamp(max=2**32 - 1).cpu().numpy().astype(np.uint32)
        at = torch.empty((hi - lo, 2), dtype=torch.int32, device=DEV)
        aliases[bj] = (ne.ne_build_neg_alias(deg_blk, lo, at), at)
    t = make_tables(V, d, K, B, seed)
    lrs = [0.025, 0.024, 0.023, 0.022, 0.021, 0.020]
    runs, base = [], 0
    for (bi, bj), same in buckets:
        runs.append((aliases[bj][0], bp.pairs[same[0][0]:same[0][0] + 3 * B], base))
        base += 3 * B
    ne.ne_train_runs(t, runs, B, K, lrs)
    torch.cuda.synchronize()
    # rows to compare: a sample of the rows the six batches name, and rows they do not name
    named_x = torch.unique(torch.cat([r[1][:, 0] for r in runs]).long())
    named_c = torch.unique(torch.cat([r[1][:, 1] for r in runs]).long())
    sx = named_x[torch.from_numpy(rng.choice(named_x.numel(), 20000, replace=False)).to(DEV)]
    sc = named_c[torch.from_numpy(rng.choice(named_c.numel(), 20000, replace=False)).to(DEV)]
    fused_x, fused_c = t.vertex[sx].clone(), t.context[sc].clone()
    # the same batches, one call each, from the same initial tables, each against the oracle
    t2 = ne.ne_create_tables(t.vertex, t.context, seed, init=True, max_batch=B, max_negatives=K, workspace=t.workspace)
    k = 0
    for (bi, bj), same in buckets:
        for (s, n, _, _) in same:
            sampled_row_check(t2, aliases[bj][0], bp.pairs[s:s + n], K, lrs[k], k * B, 128, rng)
            k += 1
    ex = rowwise_rel_err(fused_x.cpu().numpy(), t.vertex[sx].cpu().numpy())
    ec = rowwise_rel_err(fused_c.cpu().numpy(), t.context[sc].cpu().numpy())
    say(f"  one ne_train_runs call against one call per batch: row error X {ex:.2e} C {ec:.2e} on {sx.numel()} + {sc.numel()} named rows")
    assert ex <= 1e-5 and ec <= 1e-5
    assert not torch.equal(fused_x, torch.zeros_like(fused_x))


def test_maximum_batch_size():
    """One batch of NE_MAX_BATCH pairs (2^22; 29 M row references, 67 M hash positions in use) through ne_train_batch
    and a second one through ne_train_block, every element against the oracle.  A small dimension keeps the
    per-position delta slots (capacity x dim x 4 bytes) and the oracle's time small.

    The ids are heavy-tailed and clamped to the id range, so the last row collects the tail: 3.5 % of the pairs
    name it as their source, and the hottest context row is named 4e5 times.  A row that n references of one
    batch name has its n deltas added one by one in fp32 (atomic adds into the row's slot), so its error is
    bounded by n * 2^-24 of the summed magnitudes, and the bound is approached when many contributions are
    identical (same source row against the same context row: the rounding errors then all point the same way;
    1.6e-4 of the row was measured on the hottest row here).  The bar per row is therefore max(1e-4, n_r * 2^-24):
    1e-4 for every row named up to 1677 times, the accumulation bound beyond."""
    V, d, K, B, seed = 3_000_000, 8, 5, ne.NE_MAX_BATCH, 9
    say(f"maximum batch: B={B} V={V} d={d} K={K}; workspace {ne.ne_workspace_bytes(d, B, K) / 2**30:.1f} GiB")
    rng = np.random.default_rng(0)
    deg = (rng.pareto(1.0, V) * 3).astype(np.uint32) + 1
    pairs = np.minimum((rng.pareto(0.9, (2 * B, 2)) * V / 40).astype(np.int64), V - 1).astype(np.int32)
    t = make_tables(V, d, K, B, seed)
    t.context.copy_(torch.randn((V, d), generator=torch.Generator().manual_seed(1)).to(DEV) * 0.1)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at)
    thr, al, _ = oracle.build_alias(deg)
    Xo, Co = t.vertex.cpu().numpy(), t.context.cpu().numpy()
    pd = torch.from_numpy(pairs).to(DEV)
    neg = torch.empty((B, K), dtype=torch.int32, device=DEV)
    for it, call in enumerate(("ne_train_batch", "ne_train_block")):
        p = pd[it * B:(it + 1) * B]
        if it == 0:
            ne.ne_train_batch(t, alias, p, K, 0.01, it * B, neg)
        else:
            ne.ne_train_block(t, alias, p, B, K, [0.01], it * B, neg)
        torch.cuda.synchronize()
        negs = oracle.sample_negatives(seed, it * B, B, K, thr, al)
        assert np.array_equal(neg.cpu().numpy(), negs)
        pn = pairs[it * B:(it + 1) * B]
        oracle.train_batch(Xo, Co, pn, negs, 0.01)
        named = {"X": np.bincount(pn[:, 0], minlength=V),
                 "C": np.bincount(pn[:, 1], minlength=V) + np.bincount(negs.reshape(-1), minlength=V)}
        for name, got, want in (("X", t.vertex.cpu().numpy(), Xo), ("C", t.context.cpu().numpy(), Co)):
            err = np.abs(got.astype(np.float64) - want).max(axis=1)
            den = np.abs(want.astype(np.float64)).max(axis=1)
            live = den > 0
            rel = np.zeros(V); rel[live] = err[live] / den[live]
            n = named[name]
            bar = np.maximum(1e-4, n * 2.0**-24)
            worst = int(np.argmax(rel / bar))
            few = n <= 1677
            say(f"  {call} {name}: rows named <= 1677 times: max row error {rel[few].max():.2e}; oftener ({int((~few).sum())} rows, "
                f"up to {int(n.max())} times): max {rel[~few].max() if (~few).any() else 0.0:.2e}; closest to its bar: row {worst} "
                f"named {int(n[worst])} times, error {rel[worst]:.2e} of bar {bar[worst]:.2e}")
            assert (rel <= bar).all()
            assert rel[few].max() <= 1e-4
        t.vertex.copy_(torch.from_numpy(Xo)); t.context.copy_(torch.from_numpy(Co))


def test_config4_sampled_rows():
    say("config 4: 20M nodes, d=512, K=10, B=32768")
    V, d, K, B, seed = 20_000_000, 512, 10, 32768, 3
    rng = np.random.default_rng(1)
    degree = wl.rmat_degrees(V, 80_000_000, seed, device=DEV)           # a fifth of the edges: same shape, less set-up
    pairs = wl.rmat_pairs(V, 3 * B, seed, device=DEV)
    t = make_tables(V, d, K, B, seed)
    deg = degree.clamp(max=2**32 - 1).cpu().numpy().astype(np.uint32)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at)
    thr, al, _ = oracle.build_alias(deg)
    for k in range(3):                                                  # from the initial tables, then from trained ones
        if k == 2:       # the last batch through the per-reference lists, which are off by default at this size
            ne.ne_set_tuning(t, 8, 2)
        neg = sampled_row_check(t, alias, pairs[k * B:(k + 1) * B], K, 0.025, k * B, 192, rng)
        want = oracle.sample_negatives(seed, k * B, 2048, K, thr, al)
        assert np.array_equal(neg[:2048].cpu().numpy(), want)


def test_config5_whole_batch_on_compacted_rows():
    """Config 5 at full size (50 M nodes, 102 GB of tables).  A batch touches at most 2 B + N rows, so the
    oracle runs the whole batch on a compact copy of exactly those rows (ids renumbered) and every touched row
    is compared; a sample of untouched rows must stay bit-identical."""
    say("config 5: 50M nodes, d=256, B=8192, N=1024 shared negatives")
    V, d, B, N, seed = 50_000_000, 256, 8192, 1024, 4
    abc = (0.65, 0.15, 0.15)
    rng = np.random.default_rng(2)
    degree = wl.rmat_degrees(V, 200_000_000, seed, abc, device=DEV)     # a fifth of the edges
    pairs = wl.rmat_pairs(V, 2 * B, seed, abc, device=DEV)
    vertex = torch.empty((V, d), dtype=torch.float32, device=DEV)
    context = torch.empty((V, d), dtype=torch.float32, device=DEV)
    t = ne.ne_create_tables(vertex, context, seed, init=True)
    context.normal_(0.0, 0.08)                                          # a zero context table would score every pair 0
    vertex.mul_(30.0)
    deg = degree.clamp(max=2**32 - 1).cpu().numpy().astype(np.uint32)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at)
    thr, al, _ = oracle.build_alias(deg)
    ws = torch.empty(ne.ne_shared_workspace_bytes(d, B, N), dtype=torch.uint8, device=DEV)
    neg_dev = torch.empty(N, dtype=torch.int32, device=DEV)
    loss_dev = torch.zeros((), dtype=torch.float64, device=DEV)
    lr, scale = 0.025, 5.0 / N
    for it in range(2):
        p = pairs[it * B:(it + 1) * B]
        negs = oracle.sample_shared_negatives(seed, it, N, thr, al)
        negs_t = torch.from_numpy(negs).to(DEV).long()
        xs, xinv = torch.unique(p[:, 0].long(), return_inverse=True)
        cs, cinv = torch.unique(torch.cat([p[:, 1].long(), negs_t]), return_inverse=True)
        n = max(xs.numel(), cs.numel())
        Xm = np.zeros((n, d), np.float32); Cm = np.zeros((n, d), np.float32)
        Xm[: xs.numel()] = vertex[xs].cpu().numpy()
        Cm[: cs.numel()] = context[cs].cpu().numpy()
        Xb, Cb = Xm.copy(), Cm.copy()
        mp = np.stack([xinv.cpu().numpy(), cinv[:B].cpu().numpy()], axis=1).astype(np.int32)
        mn = np.ascontiguousarray(cinv[B:].cpu().numpy().astype(np.int32))
        probe = torch.from_numpy(rng.integers(0, V, 4096)).to(DEV)
        probe_c, probe_x = probe[~torch.isin(probe, cs)], probe[~torch.isin(probe, xs)]
        before_c, before_x = context[probe_c].clone(), vertex[probe_x].clone()
        loss_dev.zero_()
        ne.ne_train_batch_shared(t, alias, p, N, lr, scale, it, ws, neg_dev, loss_dev)
        torch.cuda.synchronize()
        assert np.array_equal(neg_dev.cpu().numpy(), negs)
        loss_o = oracle.train_batch_shared(Xm, Cm, mp, mn, lr, scale, bf16_inputs=True)
        assert abs(loss_dev.item() - loss_o) <= 1e-4 * loss_o
        gx, gc = vertex[xs].cpu().numpy(), context[cs].cpu().numpy()
        def derr(before, got, want):
            dg, do = got.astype(np.float64) - before, want.astype(np.float64) - before
            return np.abs(dg - do).max() / np.abs(do).max()
        ex, ec = derr(Xb[: xs.numel()], gx, Xm[: xs.numel()]), derr(Cb[: cs.numel()], gc, Cm[: cs.numel()])
        say(f"  batch {it}: {xs.numel()} + {cs.numel()} touched rows, delta err X {ex:.2e} C {ec:.2e}, loss/pair {loss_o / B:.4f}")
        assert ex <= 2e-4 and ec <= 2e-4
        assert torch.equal(context[probe_c], before_c) and torch.equal(vertex[probe_x], before_x)


def test_config2_walk_batches_full_compare():
    """Config 2's graph trained straight from its walks (ne_train_walks): 3 batches of 170 walks of length 80,
    window 5, in the fused launch configuration; negatives bit-exact and every table element against the oracle."""
    say("config 2 graph, walk batches: 1M nodes, 170 walks x 80 per batch, window 5")
    V, d, K, seed, L, win, wpb, nb = 1_000_000, 128, 5, 1, 80, 5, 170, 3
    g = wl.build_graph(V, wl.rmat_edges(V, 20_000_000, seed, device=DEV))
    starts = torch.nonzero(g.degree > 0).reshape(-1)
    starts = starts[torch.randperm(starts.numel(), generator=torch.Generator(device=DEV).manual_seed(3), device=DEV)[: nb * wpb]]
    walks = wl.random_walks(g, starts, L, seed).to(torch.int32).contiguous()
    deg = g.degree.cpu().numpy().astype(np.uint32)
    del g
    R = 1 + win * (K + 1)
    t = make_tables(V, d, K, -(-(wpb * L * R) // (K + 2)), seed)
    t.context.copy_(torch.randn((V, d), generator=torch.Generator().manual_seed(2)).to(DEV) * 0.05)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at)
    thr, al, _ = oracle.build_alias(deg)
    Xo, Co = t.vertex.cpu().numpy(), t.context.cpu().numpy()
    lrs = [0.025, 0.02, 0.015]
    neg_out = torch.full((nb * wpb, L, win, K), -1, dtype=torch.int32, device=DEV)
    ne.ne_train_walks(t, alias, walks, wpb, win, K, lrs, 0, neg_out)
    torch.cuda.synchronize()
    wn = walks.cpu().numpy()
    got = neg_out.cpu().numpy().reshape(-1, K)
    for b in range(nb):
        part = np.ascontiguousarray(wn[b * wpb:(b + 1) * wpb])
        pairs, sample = oracle.walk_pairs(part, win)
        first = b * wpb * L * win
        neg_all = oracle.sample_negatives(seed, first, wpb * L * win, K, thr, al)
        neg = np.ascontiguousarray(neg_all[sample])
        assert np.array_equal(got[first + sample], neg)
        oracle.train_batch(Xo, Co, pairs, neg, lrs[b])
    ex = rowwise_rel_err(t.vertex.cpu().numpy(), Xo)
    ec = rowwise_rel_err(t.context.cpu().numpy(), Co)
    say(f"  rowwise err X {ex:.2e} C {ec:.2e}")
    assert ex <= 3e-4 and ec <= 3e-4       # three batches
