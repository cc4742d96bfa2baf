"""ne_score_pairs against the oracle, and the link-prediction protocol of Sec. V-B end to end on a synthetic
planted-partition network (the paper's YouTube / Hyperlink-PLD data do not ship here): embeddings trained on
90 % of the edges must rank the held-out edges above random non-edges."""
import numpy as np
import pytest
import torch

import oracle
import paper_2005_13789_amd as ne
from paper_2005_13789_amd import linkpred as lp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("V,d,n", [(300, 128, 5000), (50, 4, 33), (1000, 1024, 257), (64, 72, 0)])
def test_score_pairs_matches_oracle(V, d, n):
    say(f"score pairs V={V} d={d} n={n}")
    rng = np.random.default_rng(V + d)
    X = rng.normal(0, 0.5, (V, d)).astype(np.float32)
    C = rng.normal(0, 0.5, (V, d)).astype(np.float32)
    pairs = rng.integers(0, V, (n, 2)).astype(np.int32)
    vertex, context = torch.from_numpy(X).to(DEV), torch.from_numpy(C).to(DEV)
    t = ne.ne_create_tables(vertex, context, 0, init=False)
    out = torch.full((max(n, 1),), 7.0, dtype=torch.float32, device=DEV)
    for flag in (True, False):
        ne.ne_score_pairs(t, torch.from_numpy(pairs).to(DEV), out, flag)
        torch.cuda.synchronize()
        want = oracle.score_pairs(X, C, pairs, flag)
        got = out.cpu().numpy()[:n].astype(np.float64)
        # fp32 products summed in a tree over d terms: error <= d * 2^-24 * sum |a_k b_k|
        bound = d * 2.0 ** -24 * np.abs(X[pairs[:, 0]].astype(np.float64) * (C if flag else X)[pairs[:, 1]]).sum(axis=1)
        assert np.all(np.abs(got - want) <= bound + 1e-30)
    if n == 0:
        assert out.item() == 7.0                     # nothing written
    assert torch.equal(vertex.cpu(), torch.from_numpy(X)) and torch.equal(context.cpu(), torch.from_numpy(C))


def planted_partition(V, communities, inside, outside, seed):
    """Each node draws `inside` neighbours in its own community and `outside` anywhere."""
    rng = np.random.default_rng(seed)
    size = V // communities
    u = np.repeat(np.arange(V), inside)
    v = (u // size) * size + rng.integers(0, size, u.size)
    uo = np.repeat(np.arange(V), outside)
    vo = rng.integers(0, V, uo.size)
    return np.stack([np.concatenate([u, uo]), np.concatenate([v, vo])], axis=1)


# The per-sample mode loses no update (rows shared inside a call take atomic adds), so it trains at the same
# call size as the exact step.
@pytest.mark.parametrize("mode,batch", [("sync", 4096), ("async", 4096), ("walks", 4096)])
def test_link_prediction_auc_on_planted_partition(mode, batch):
    V = 4000
    edges = planted_partition(V, communities=40, inside=10, outside=1, seed=1)
    train, test = lp.split_edges(edges, 0.10, seed=2)
    say(f"link prediction ({mode}): {train.shape[0]} training edges, {test.shape[0]} held out")
    all_edges = np.concatenate([train, test])
    tables, alias = lp.train(train, V, dim=64, epochs=10, negatives=5, batch=batch, lr0=0.025, walk_length=40, window=5,
                             seed=3, mode=mode, device=DEV)
    assert torch.isfinite(tables.vertex).all() and torch.isfinite(tables.context).all()
    auc_vc = lp.evaluate(tables, V, all_edges, test, seed=4, second_from_context=True)
    auc_vv = lp.evaluate(tables, V, all_edges, test, seed=4, second_from_context=False)
    say(f"  AUC vertex.context {auc_vc:.4f}   vertex.vertex {auc_vv:.4f}")
    # untrained tables rank at chance
    fresh_v = torch.empty_like(tables.vertex); fresh_c = torch.empty_like(tables.context)
    fresh = ne.ne_create_tables(fresh_v, fresh_c, 3, init=True)
    fresh_c.copy_(torch.randn_like(fresh_c) * 0.01)
    auc0 = lp.evaluate(fresh, V, all_edges, test, seed=4)
    say(f"  AUC before training {auc0:.4f}")
    assert abs(auc0 - 0.5) < 0.05
    # one edge in eleven of this network is random and cannot be predicted: the ceiling is about 0.955
    assert auc_vc > 0.9 and auc_vv > 0.9


def test_command_line_on_an_edge_list_file(tmp_path, capsys):
    import json
    edges = planted_partition(1000, communities=10, inside=8, outside=1, seed=5)
    f = tmp_path / "edges.txt"
    f.write_text("# u v\n" + "\n".join(f"{a + 100} {b + 100}" for a, b in edges.tolist()) + "\n")    # ids need not start at 0
    assert lp.main([str(f), "--test-fraction", "0.1", "--dim", "32", "--epochs", "8", "--batch", "2048", "--mode", "walks"]) == 0
    out = json.loads(capsys.readouterr().out.strip().splitlines()[-1])
    print(out, flush=True)
    assert out["nodes"] == 1000 and out["auc_vertex_context"] > 0.85
