"""ne_train_runs: a sequence of runs (sample blocks with their own negative-sampling tables) in one call, the
id-only work of a run's first batch riding in the previous run's last batch.  Against the CPU oracle batch by
batch (negatives bit-exact, tables row-wise), and against one ne_train_block call per run."""
import numpy as np
import pytest
import torch

import oracle
import paper_2005_13789_amd as ne
from parity_util import rowwise_rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make(V, d, B, K, seed):
    vertex = torch.empty((V, d), dtype=torch.float32, device=DEV)
    context = torch.empty((V, d), dtype=torch.float32, device=DEV)
    ws = torch.empty(ne.ne_workspace_bytes(d, B, K), dtype=torch.uint8, device=DEV)
    t = ne.ne_create_tables(vertex, context, seed, init=True, max_batch=B, max_negatives=K, workspace=ws)
    context.copy_(torch.randn((V, d), generator=torch.Generator().manual_seed(seed)).to(DEV) * 0.05)
    return t


@pytest.mark.parametrize("sizes", [(2500, 1024, 1, 3000), (700,), (1024, 1024), (5, 0, 9, 2048, 0)])
def test_runs_match_oracle_and_per_run_calls(sizes):
    print(f"runs of {sizes} pairs", flush=True)
    V, d, K, B, seed, grid = 40000, 64, 5, 1024, 8, 4
    block = V // grid
    rng = np.random.default_rng(len(sizes))
    deg = (rng.pareto(1.0, V) * 3).astype(np.uint32) + 1
    # run r trains source block r % 4 against context block (r + 1) % 4, negatives from that context block only
    aliases, tables_o = [], []
    for j in range(grid):
        at = torch.empty((block, 2), dtype=torch.int32, device=DEV)
        aliases.append(ne.ne_build_neg_alias(deg[j * block:(j + 1) * block], j * block, at))
        tables_o.append(oracle.build_alias(deg[j * block:(j + 1) * block])[:2])
    runs, lrs, base = [], [], 0
    for r, n in enumerate(sizes):
        bi, bj = r % grid, (r + 1) % grid
        src = bi * block + np.minimum((rng.pareto(0.8, n) * block / 30).astype(np.int64), block - 1)
        ctx = bj * block + np.minimum((rng.pareto(0.8, n) * block / 30).astype(np.int64), block - 1)
        pairs = np.stack([src, ctx], axis=1).astype(np.int32)
        runs.append((bj, pairs, base))
        lrs += [0.03 / (1 + len(lrs) + i) for i in range(-(-n // B))]
        base += n + 17                       # sample indices need not be contiguous across runs
    chained, single = make(V, d, B, K, seed), make(V, d, B, K, seed)
    Xo, Co = chained.vertex.cpu().numpy(), chained.context.cpu().numpy()
    negs = [torch.full((max(p.shape[0], 1), K), -1, dtype=torch.int32, device=DEV) for _, p, _ in runs]
    dev_pairs = [torch.from_numpy(p).to(DEV) for _, p, _ in runs]
    ne.ne_train_runs(chained, [(aliases[bj], dp, sb, ng) for (bj, _, sb), dp, ng in zip(runs, dev_pairs, negs)], B, K, lrs)
    at = 0
    for (bj, p, sb), dp in zip(runs, dev_pairs):
        nb = -(-p.shape[0] // B)
        ne.ne_train_block(single, aliases[bj], dp, B, K, lrs[at:at + nb] or [0.0], sb)
        at += nb
    torch.cuda.synchronize()
    ex = rowwise_rel_err(chained.vertex.cpu().numpy(), single.vertex.cpu().numpy())
    ec = rowwise_rel_err(chained.context.cpu().numpy(), single.context.cpu().numpy())
    print(f"  chained vs one call per run: row error X {ex:.2e} C {ec:.2e}", flush=True)
    assert ex <= 1e-5 and ec <= 1e-5
    at = 0
    for (bj, p, sb), ng in zip(runs, negs):
        thr, al = tables_o[bj]
        for first in range(0, p.shape[0], B):
            pb = np.ascontiguousarray(p[first:first + B])
            neg = oracle.sample_negatives(seed, sb + first, pb.shape[0], K, thr, al, bj * block)
            assert np.array_equal(ng[first:first + pb.shape[0]].cpu().numpy(), neg)
            oracle.train_batch(Xo, Co, pb, neg, lrs[at])
            at += 1
    ox = rowwise_rel_err(chained.vertex.cpu().numpy(), Xo)
    oc = rowwise_rel_err(chained.context.cpu().numpy(), Co)
    print(f"  against the oracle after {at} batches: row error X {ox:.2e} C {oc:.2e}", flush=True)
    assert ox <= min(1e-4 * max(at, 1), 1e-3) and oc <= min(1e-4 * max(at, 1), 1e-3)


def test_runs_argument_errors():
    V, d, K, B = 1000, 32, 2, 64
    t = make(V, d, B, K, 1)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(np.ones(V, np.uint32), 0, at)
    pairs = torch.zeros((100, 2), dtype=torch.int32, device=DEV)
    before = t.vertex.clone()
    ne.ne_train_runs(t, [], B, K, [])                                   # no runs: no-op
    ne.ne_train_runs(t, [(alias, pairs[:0], 0)], B, K, [])              # an empty run: skipped
    with pytest.raises(TypeError):
        ne.ne_train_runs(t, [(alias, pairs, 0)], B, K, [0.1])           # two batches, one learning rate
    with pytest.raises(ne.NeError):
        ne.ne_train_runs(t, [(None, pairs, 0)], B, K, [0.1, 0.1])       # K > 0 without an alias table
    with pytest.raises(ne.NeError):
        ne.ne_train_runs(t, [(alias, pairs, 0)], 2 * B, K, [0.1])       # B beyond the workspace
    with pytest.raises(ne.NeError):
        ne.ne_train_runs(t, [(alias, pairs, 0)], B, K, [0.1, float("nan")])
    torch.cuda.synchronize()
    assert torch.equal(t.vertex, before)
