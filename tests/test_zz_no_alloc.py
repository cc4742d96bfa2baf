"""ne_train_batch_shared_static (the entry point that allocates nothing: its scratch is a static per-GPU
array inside the library) against ne_train_batch_shared (scratch from the caller) through the C ABI.

Same kernels, same inputs: the two results may differ only in the order of the fp32 atomic adds on rows
named more than once, so the updates must agree far inside the shared-negative mode's parity bar
(|d_static - d_workspace|_inf <= 2e-4 |d_workspace|_inf per table; measured ~1e-6), negative ids and rows
the batch does not name bit for bit.  Two calls in a row on the same GPU, the second with a smaller input:
the array keeps the first call's contents and the second call must not depend on them.
"""
import ctypes

import numpy as np
import pytest
import torch

import paper_2005_13789_amd as ne

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def raw_static(L, t, alias, pairs, N, lr, scale, batch_index, neg_out, loss):
    """The C entry point itself, through ctypes, with plain pointers."""
    return L.ne_train_batch_shared_static(t.handle, alias.handle, pairs.data_ptr(), int(pairs.shape[0]), N, lr, scale,
                                          batch_index, neg_out.data_ptr(), loss.data_ptr(),
                                          int(torch.cuda.current_stream().cuda_stream))


def delta_err(before, got, want):
    dg = got.astype(np.float64) - before.astype(np.float64)
    dw = want.astype(np.float64) - before.astype(np.float64)
    return np.abs(dg - dw).max() / max(np.abs(dw).max(), 1e-30)


def test_static_scratch_matches_workspace_entry_point():
    L = ne.lib()
    V, d, seed = 6000, 128, 21
    rng = np.random.default_rng(4)
    deg = (rng.pareto(1.0, V) * 2).astype(np.uint32) + 1
    X = rng.normal(0, 1.5 / np.sqrt(d), (V, d)).astype(np.float32)
    C = rng.normal(0, 1.5 / np.sqrt(d), (V, d)).astype(np.float32)
    side = {}
    for name in ("workspace", "static"):
        vertex, context = torch.from_numpy(X).to(DEV), torch.from_numpy(C).to(DEV)
        t = ne.ne_create_tables(vertex, context, seed, init=False)
        at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
        alias = ne.ne_build_neg_alias(deg, 0, at)
        side[name] = (vertex, context, t, alias, at)
    # first call: several row tiles and a ragged tail; second call: smaller B and N, other layout of the scratch
    for call, (B, N) in enumerate([(3000, 512), (700, 128)]):
        say(f"static scratch call {call}: d={d} B={B} N={N}")
        assert ne.ne_shared_workspace_bytes(d, B, N) <= ne.NE_SHARED_STATIC_SCRATCH_BYTES
        pairs = np.minimum((rng.pareto(0.8, (B, 2)) * V / 50).astype(np.int64), V - 1).astype(np.int32)
        pd = torch.from_numpy(pairs).to(DEV)
        lr, scale = 0.05, 5.0 / N
        before_x, before_c = side["workspace"][0].cpu().numpy(), side["workspace"][1].cpu().numpy()
        out = {}
        for name in ("workspace", "static"):
            vertex, context, t, alias, _ = side[name]
            neg = torch.empty(N, dtype=torch.int32, device=DEV)
            loss = torch.zeros((), dtype=torch.float64, device=DEV)
            if name == "workspace":
                ws = torch.empty(ne.ne_shared_workspace_bytes(d, B, N), dtype=torch.uint8, device=DEV)
                ne.ne_train_batch_shared(t, alias, pd, N, lr, scale, 5 + call, ws, neg, loss)
            else:
                rc = raw_static(L, t, alias, pd, N, lr, scale, 5 + call, neg, loss)
                assert rc == ne.NE_OK, ne.ne_last_error()
            torch.cuda.synchronize()
            out[name] = (vertex.cpu().numpy(), context.cpu().numpy(), neg.cpu().numpy(), loss.item())
        xw, cw, nw, lw = out["workspace"]
        xs, cs, ns, ls = out["static"]
        assert np.array_equal(nw, ns)
        assert abs(lw - ls) <= 1e-9 * abs(lw), (lw, ls)
        ex, ec = delta_err(before_x, xs, xw), delta_err(before_c, cs, cw)
        say(f"  delta err vs workspace entry point: X {ex:.2e} C {ec:.2e}; loss {ls / B:.4f}")
        assert ex <= 2e-4 and ec <= 2e-4
        assert ex <= 1e-5 and ec <= 1e-5          # same kernels: only the order of atomic adds may differ
        touched_x = np.zeros(V, bool); touched_x[pairs[:, 0]] = True
        touched_c = np.zeros(V, bool); touched_c[pairs[:, 1]] = True; touched_c[nw] = True
        assert np.array_equal(xs[~touched_x].view(np.uint32), before_x[~touched_x].view(np.uint32))
        assert np.array_equal(cs[~touched_c].view(np.uint32), before_c[~touched_c].view(np.uint32))
        assert touched_x.sum() > 0 and not np.array_equal(xs, before_x)
        # continue both sides from the same state
        side["static"][0].copy_(side["workspace"][0]); side["static"][1].copy_(side["workspace"][1])


def test_static_scratch_rejects_shapes_beyond_its_size():
    L = ne.lib()
    V, d = 500, 256
    vertex = torch.zeros((V, d), dtype=torch.float32, device=DEV)
    context = torch.zeros((V, d), dtype=torch.float32, device=DEV)
    t = ne.ne_create_tables(vertex, context, 0, init=False)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(np.ones(V, np.uint32), 0, at)
    B, N = 8192, 1024
    assert ne.ne_shared_workspace_bytes(d, B, N) > ne.NE_SHARED_STATIC_SCRATCH_BYTES
    pairs = torch.zeros((B, 2), dtype=torch.int32, device=DEV)
    neg = torch.empty(N, dtype=torch.int32, device=DEV)
    loss = torch.zeros((), dtype=torch.float64, device=DEV)
    rc = raw_static(L, t, alias, pairs, N, 0.1, 0.1, 0, neg, loss)
    assert rc == ne.NE_ERR_ARG
    assert "static scratch" in ne.ne_last_error()
    with pytest.raises(ne.NeError):
        ne.ne_train_batch_shared_static(t, alias, pairs, 100, 0.1, 0.1, 0)        # N not a multiple of 128
    ne.ne_train_batch_shared_static(t, alias, pairs[:0], 128, 0.1, 0.1, 0)        # empty batch: no-op
    torch.cuda.synchronize()
    assert not vertex.any() and not context.any()
