"""Helpers shared by the GPU parity tests: device set-up through the binding, error metrics."""
import numpy as np
import torch

import oracle
import paper_2005_13789_amd as ne


def rowwise_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max over rows r with |want_r|_inf > 0 of |got_r - want_r|_inf / |want_r|_inf."""
    g = got.astype(np.float64)
    w = want.astype(np.float64)
    num = np.abs(g - w).max(axis=1)
    den = np.abs(w).max(axis=1)
    live = den > 0
    if not live.any():
        return float(num.max()) if num.size else 0.0
    return float((num[live] / den[live]).max())


def table_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    w = np.abs(want.astype(np.float64)).max()
    return float(np.abs(got.astype(np.float64) - want.astype(np.float64)).max() / (w if w > 0 else 1.0))


class GpuModel:
    """Tables + alias + staging on cuda:0, driven only through the C-ABI binding."""

    def __init__(self, V, d, seed, degree, K, max_B, base=0, n_alias=None, init=True, X=None, C=None):
        dev = torch.device("cuda:0")
        self.V, self.d, self.K, self.seed = V, d, K, seed
        self.vertex = torch.empty((V, d), dtype=torch.float32, device=dev)
        self.context = torch.empty((V, d), dtype=torch.float32, device=dev)
        if X is not None:
            self.vertex.copy_(torch.from_numpy(X))
            self.context.copy_(torch.from_numpy(C))
            init = False
        self.workspace = torch.empty(ne.ne_workspace_bytes(d, max(max_B, 1), K), dtype=torch.uint8, device=dev)
        self.tables = ne.ne_create_tables(self.vertex, self.context, seed, init=init, max_batch=max(max_B, 1),
                                          max_negatives=K, workspace=self.workspace)
        self.alias = None
        if degree is not None:
            n = len(degree)
            self.alias_table = torch.empty((n, 2), dtype=torch.int32, device=dev)
            self.alias = ne.ne_build_neg_alias(np.asarray(degree, dtype=np.uint32), base, self.alias_table)
        self.neg_out = torch.empty((max(max_B, 1), max(K, 1)), dtype=torch.int32, device=dev)
        self.loss = torch.zeros((), dtype=torch.float64, device=dev)

    def train(self, pairs_dev, lr, sample_base, want_neg=True):
        B = pairs_dev.shape[0]
        ne.ne_train_batch(self.tables, self.alias, pairs_dev, self.K, lr, sample_base,
                          self.neg_out if want_neg else None)
        if want_neg:
            return self.neg_out[:B, :self.K].cpu().numpy() if self.K > 0 else np.zeros((B, 0), np.int32)
        return None

    def loss_sum(self, pairs_dev, sample_base):
        self.loss.zero_()
        ne.ne_eval_loss(self.tables, self.alias, pairs_dev, self.K, sample_base, self.loss, self.neg_out)
        return float(self.loss.item())

    def host_tables(self):
        torch.cuda.synchronize()
        return self.vertex.cpu().numpy(), self.context.cpu().numpy()


def oracle_negatives(seed, sample_base, B, K, degree, base=0):
    if K == 0:
        return np.zeros((B, 0), dtype=np.int32)
    thr, alias, _ = oracle.build_alias(np.asarray(degree, dtype=np.uint32))
    return oracle.sample_negatives(seed, sample_base, B, K, thr, alias, base)
