"""Sample batches prefetched from pinned host memory while training (Sec. IV-A pipeline, single-GPU part):
ne_train_block_pinned against the CPU oracle on the same batches (negatives bit-exact, tables row-wise within
1e-4 per batch), and against ne_train_block on resident pairs."""
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


@pytest.mark.parametrize("n", [11 * 1024 + 300, 1024, 700, 2 * 1024, 3 * 1024 + 1])
def test_pinned_block_equals_resident_block(n):
    """ne_train_block_pinned: the prefetch rides inside the training launches."""
    print(f"pinned block, {n} pairs", flush=True)
    V, d, K, B = 30000, 64, 5, 1024
    rng = np.random.default_rng(n)
    deg = (rng.pareto(1.0, V) * 3).astype(np.uint32) + 1
    pairs = torch.from_numpy(((rng.pareto(0.9, (n, 2)) * V / 30).astype(np.int64) % V).astype(np.int32))
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at)
    nb = -(-n // B)
    lrs = [0.02 / (1 + 0.1 * b) for b in range(nb)]
    resident, pinned = make(V, d, B, K, 4), make(V, d, B, K, 4)
    Xo, Co = pinned.vertex.cpu().numpy(), pinned.context.cpu().numpy()
    neg_r = torch.empty((n, K), dtype=torch.int32, device=DEV)
    neg_p = torch.empty((n, K), dtype=torch.int32, device=DEV)
    ne.ne_train_block(resident, alias, pairs.to(DEV), B, K, lrs, 500, neg_r)
    staging = torch.full((3, B, 2), -1, dtype=torch.int32, device=DEV)
    ne.ne_train_block_pinned(pinned, alias, pairs.pin_memory(), B, K, lrs, 500, staging, neg_p)
    torch.cuda.synchronize()
    assert torch.equal(neg_r, neg_p)
    ex = rowwise_rel_err(pinned.vertex.cpu().numpy(), resident.vertex.cpu().numpy())
    ec = rowwise_rel_err(pinned.context.cpu().numpy(), resident.context.cpu().numpy())
    print(f"  row error X {ex:.2e} C {ec:.2e}", flush=True)
    assert ex <= 1e-5 and ec <= 1e-5
    # the oracle on the same batches
    thr, al, _ = oracle.build_alias(deg)
    pn = pairs.numpy()
    for b in range(nb):
        p = np.ascontiguousarray(pn[b * B:(b + 1) * B])
        neg = oracle.sample_negatives(4, 500 + b * B, p.shape[0], K, thr, al)
        assert np.array_equal(neg_p[b * B:b * B + p.shape[0]].cpu().numpy(), neg)
        oracle.train_batch(Xo, Co, p, neg, lrs[b])
    ox = rowwise_rel_err(pinned.vertex.cpu().numpy(), Xo)
    oc = rowwise_rel_err(pinned.context.cpu().numpy(), Co)
    print(f"  against the oracle after {nb} batches: row error X {ox:.2e} C {oc:.2e}", flush=True)
    assert ox <= min(1e-4 * nb, 1e-3) and oc <= min(1e-4 * nb, 1e-3)
    with pytest.raises(TypeError):
        ne.ne_train_block_pinned(pinned, alias, pairs, B, K, lrs, 500, staging)       # pageable host memory
