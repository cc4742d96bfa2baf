"""The training calls are kernel launches only (no memsets, no synchronisation, no allocation), so a caller
may capture them in a HIP graph.  A captured run of batches is replayed several times, with eager work and
synchronisation between the replays, and every replay is checked against the same calls made eagerly."""
import numpy as np
import pytest
import torch

import paper_2005_13789_amd as ne
from parity_util import rowwise_rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def make(V, d, B, K, seed):
    vertex = torch.empty((V, d), dtype=torch.float32, device=DEV)
    context = torch.empty((V, d), dtype=torch.float32, device=DEV)
    ws = torch.empty(ne.ne_workspace_bytes(d, B, K), dtype=torch.uint8, device=DEV)
    t = ne.ne_create_tables(vertex, context, seed, init=True, max_batch=B, max_negatives=K, workspace=ws)
    context.copy_(torch.randn((V, d), generator=torch.Generator().manual_seed(seed)).to(DEV) * 0.05)
    return t


def test_captured_block_replays_match_eager_calls():
    V, d, B, K, batches, replays = 20000, 128, 2048, 5, 3, 4
    say(f"graph capture: exact step, {batches} batches x {replays} replays")
    rng = np.random.default_rng(0)
    deg = (rng.pareto(1.0, V) * 3).astype(np.uint32) + 1
    pairs = torch.from_numpy(np.minimum((rng.pareto(0.9, (batches * B, 2)) * V / 40).astype(np.int64), V - 1).astype(np.int32)).to(DEV)
    lrs = [0.02, 0.015, 0.01]
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at)
    eager, graphed = make(V, d, B, K, 5), make(V, d, B, K, 5)
    loss = torch.zeros((), dtype=torch.float64, device=DEV)

    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        snap_v, snap_c = graphed.vertex.clone(), graphed.context.clone()
        ne.ne_train_block(graphed, alias, pairs, B, K, lrs, 0)              # warm-up on the capture stream
        graphed.vertex.copy_(snap_v); graphed.context.copy_(snap_c)
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            ne.ne_train_block(graphed, alias, pairs, B, K, lrs, 0)
    torch.cuda.current_stream().wait_stream(stream)
    torch.cuda.synchronize()

    for r in range(replays):
        ne.ne_train_block(eager, alias, pairs, B, K, lrs, 0)
        graph.replay()
        torch.cuda.synchronize()
        ex = rowwise_rel_err(graphed.vertex.cpu().numpy(), eager.vertex.cpu().numpy())
        ec = rowwise_rel_err(graphed.context.cpu().numpy(), eager.context.cpu().numpy())
        say(f"  replay {r}: graph vs eager row error X {ex:.2e} C {ec:.2e}")
        assert ex <= 1e-4 and ec <= 1e-4
        # the program's own eager work between replays
        loss.zero_()
        ne.ne_eval_loss(eager, alias, pairs[:B], K, 0, loss)
        torch.cuda.synchronize()
        assert np.isfinite(loss.item())


def test_captured_shared_negative_step_replays_match_eager_calls():
    V, d, B, N, replays = 30000, 128, 3000, 256, 3
    say(f"graph capture: shared-negative step x {replays} replays")
    rng = np.random.default_rng(1)
    deg = (rng.pareto(1.0, V) * 3).astype(np.uint32) + 1
    pairs = torch.from_numpy(np.minimum((rng.pareto(0.9, (B, 2)) * V / 40).astype(np.int64), V - 1).astype(np.int32)).to(DEV)
    at = torch.empty((V, 2), dtype=torch.int32, device=DEV)
    alias = ne.ne_build_neg_alias(deg, 0, at)
    eager, graphed = make(V, d, 1, 1, 6), make(V, d, 1, 1, 6)
    ws_e = torch.empty(ne.ne_shared_workspace_bytes(d, B, N), dtype=torch.uint8, device=DEV)
    ws_g = torch.empty_like(ws_e)

    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        snap_v, snap_c = graphed.vertex.clone(), graphed.context.clone()
        ne.ne_train_batch_shared(graphed, alias, pairs, N, 0.02, 5.0 / N, 9, ws_g)   # warm-up (raises the kernel's LDS limit)
        graphed.vertex.copy_(snap_v); graphed.context.copy_(snap_c)
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            ne.ne_train_batch_shared(graphed, alias, pairs, N, 0.02, 5.0 / N, 9, ws_g)
    torch.cuda.current_stream().wait_stream(stream)
    torch.cuda.synchronize()

    for r in range(replays):
        ne.ne_train_batch_shared(eager, alias, pairs, N, 0.02, 5.0 / N, 9, ws_e)
        graph.replay()
        torch.cuda.synchronize()
        ex = rowwise_rel_err(graphed.vertex.cpu().numpy(), eager.vertex.cpu().numpy())
        ec = rowwise_rel_err(graphed.context.cpu().numpy(), eager.context.cpu().numpy())
        say(f"  replay {r}: graph vs eager row error X {ex:.2e} C {ec:.2e}")
        assert ex <= 1e-4 and ec <= 1e-4
        ws_e.random_(0, 255)                         # eager work between replays; the workspace carries nothing
        torch.cuda.synchronize()
