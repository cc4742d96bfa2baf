#!/usr/bin/env python3
"""Throughput of the SGNS training hot path on one MI355X.

A step is one ne_train_batch call (negative sampling, row gather, scoring, gradient formation and
the scatter update) on one batch of synthetic positive pairs that already reside in HBM.

Workloads (synthetic R-MAT stand-ins for the paper's graphs):
  c3  one GPU's partition at paper scale: 100 M nodes, dim 128, both tables resident (102 GB), pairs
      pre-bucketed over a 4x4 (src-block, ctx-block) grid, K=5 negatives from the ctx block.  Default:
      it is the configuration the HBM-bandwidth target is stated on.
  c2  1 M nodes / 20 M edges, walks of 80, window 5, dim 128, K=5, batch 65536.
  c4  20 M nodes, dim 512, K=10, batch 32768.
  c1  10 k nodes, dim 128, K=5, batch 4096 (the parity configuration; cache resident).
  c5  shared-negative mode: 50 M nodes (R-MAT a=0.65), dim 256, batches of 8192 pairs that share 1024
      negatives (bf16 MFMA tiles, fp32 accumulate and update); its roofline is the matrix cores'.

Prints one JSON line.  --gpus above 1 is refused: this build is single-GPU.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import paper_2005_13789_amd as ne  # noqa: E402
import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the dominant kernel come from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summaries
# under profiles/ (each scaled there by what the same counter reads for a plain copy of known size): the line
# "TRAFFIC_BYTES_PER_LAUNCH <kernel> <bytes>" of profiles/<kernel>_<workload>_hbm_counters.txt.
def traffic_bytes_per_launch(kernel: str, workload: str):
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_hbm_counters.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 3 and parts[0] == "TRAFFIC_BYTES_PER_LAUNCH" and parts[1] == kernel:
                    return float(parts[2])
    except OSError:
        pass
    return None


MFMA_BF16_PEAK_TFLOPS = 2500.0

WORKLOADS = {
    "c1": dict(V=10_000, edges=100_000, d=128, K=5, B=4096, grid=1, abc=(0.57, 0.19, 0.19), walk=(40, 5), seed=0),
    "c2": dict(V=1_000_000, edges=20_000_000, d=128, K=5, B=65536, grid=1, abc=(0.57, 0.19, 0.19), walk=(80, 5), seed=1),
    "c3": dict(V=100_000_000, edges=2_000_000_000, d=128, K=5, B=65536, grid=4, abc=(0.57, 0.19, 0.19), walk=None, seed=2),
    "c4": dict(V=20_000_000, edges=400_000_000, d=512, K=10, B=32768, grid=1, abc=(0.57, 0.19, 0.19), walk=None, seed=3,
               walk_shape=(80, 10)),
    "c5": dict(V=50_000_000, edges=1_000_000_000, d=256, K=0, B=8192, grid=1, abc=(0.65, 0.15, 0.15), walk=None, seed=4,
               shared_negatives=1024),
}


def algorithmic_bytes_per_pair(d: int, K: int) -> int:
    """Every touched row read once and written once, plus the pair and one alias entry per negative."""
    return 2 * (2 + K) * 4 * d + 8 + 8 * K


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def build_workload(name: str, n_batches: int, dev):
    w = WORKLOADS[name]
    V, d, K, B, grid, seed = w["V"], w["d"], w["K"], w["B"], w["grid"], w["seed"]
    t0 = time.time()
    if w["walk"] is not None:
        # real graph + random walks (host for the small case, device for 1 M nodes)
        gdev = "cpu" if V <= 100_000 else dev
        g = wl.build_graph(V, wl.rmat_edges(V, w["edges"], seed, w["abc"], device=gdev))
        L, win = w["walk"]
        pairs = wl.walk_pairs(g, L, win, n_batches * B, seed).to(dev)
        degree = g.degree
        del g
    else:
        degree = wl.rmat_degrees(V, w["edges"], seed, w["abc"], device=dev)
        # extra pairs so that every bucket can be cut to whole batches
        pairs = wl.rmat_pairs(V, n_batches * B + grid * grid * B, seed, w["abc"], device=dev)
    log(f"{name}: graph/pairs generated in {time.time() - t0:.1f}s")
    bp = wl.bucket_pairs(pairs, V, grid)
    sched = [s for s in wl.orthogonal_schedule(bp, B) if s[1] == B]
    if len(sched) < n_batches:
        # cycle through the schedule again (walk pairs may be reused across epochs, Sec. V-C)
        sched = (sched * (n_batches // max(len(sched), 1) + 1))
    sched = sched[:n_batches]
    return w, degree, bp, sched


def apply_tuning(args, tables):
    if args.tuning:
        list_cap, sweep = (int(v) for v in args.tuning.split(","))
        ne.ne_set_tuning(tables, list_cap, sweep)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="c3", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--repeats", type=int, default=5,
                    help="the timed region is run this many times, tables initialised again each time; the median is reported")
    ap.add_argument("--per-batch", action="store_true", help="one library call per batch (no fused prepare)")
    ap.add_argument("--per-run", action="store_true", help="one ne_train_block call per bucket run instead of one ne_train_runs call")
    ap.add_argument("--mode", default="sync", choices=["sync", "async"],
                    help="sync: exact minibatch-synchronous step (the benchmark); async: per-sample mode (shared rows updated with atomics in place)")
    ap.add_argument("--cpu-batches", type=int, default=0, help="oracle batches to time (0 = auto)")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size (experiments)")
    ap.add_argument("--subparts", type=int, default=0,
                    help="sub-part ping-pong scenario: the vertex rows of one source block live in pinned host memory "
                         "and stream through the device in this many sub-parts while training (c3 shape)")
    ap.add_argument("--pinned-pairs", action="store_true",
                    help="keep the pairs in pinned host memory: ne_train_block_pinned prefetches them inside the training "
                         "launches (the sample-batch H2D of the paper's pipeline)")
    ap.add_argument("--walks", action="store_true",
                    help="on-device augmentation scenario (walk workloads c1, c2): the same whole-walk batches through "
                         "ne_train_walks and, expanded to pairs, through ne_train_block")
    ap.add_argument("--tuning", default="", metavar="LIST_CAP,SWEEP",
                    help="override the library's automatic choices (ne_set_tuning), e.g. 0,8 or 8,2 (experiments)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run 20 plain 1 GiB device copies (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": 1 << 30, "bytes_written": 1 << 30, "copies": 20}}))
        return
    if args.subparts > 0:
        subparts_scenario(args, dev)
        return
    if args.walks:
        walks_scenario(args, dev)
        return
    name = args.workload
    if args.batch > 0:
        WORKLOADS[name] = dict(WORKLOADS[name], B=args.batch)
    n_batches = args.steps + args.warmup
    w, degree, bp, sched = build_workload(name, n_batches, dev)
    V, d, K, B, grid, seed = w["V"], w["d"], w["K"], w["B"], w["grid"], w["seed"]

    t0 = time.time()
    vertex = torch.empty((V, d), dtype=torch.float32, device=dev)
    context = torch.empty((V, d), dtype=torch.float32, device=dev)
    N = w.get("shared_negatives", 0)
    if N:
        workspace = torch.empty(ne.ne_shared_workspace_bytes(d, B, N), dtype=torch.uint8, device=dev)
    else:
        workspace = torch.empty(ne.ne_workspace_bytes(d, B, K), dtype=torch.uint8, device=dev)

    def fresh_tables():
        """Both tables initialised again on the device (vertex uniform, context zero), workspace cleared."""
        if N:
            return ne.ne_create_tables(vertex, context, seed, init=True)
        t = ne.ne_create_tables(vertex, context, seed, init=True, max_batch=B, max_negatives=K, workspace=workspace)
        apply_tuning(args, t)
        return t

    tables = fresh_tables()
    # one alias table per context block (a GPU's context partition is fixed; negatives come from it)
    block = bp.block_rows
    deg_host = degree.to(torch.int64).clamp_(max=2**32 - 1).cpu().numpy().astype(np.uint32)
    aliases = []
    for j in range(grid):
        lo, hi = j * block, min((j + 1) * block, V)
        table = torch.empty((hi - lo, 2), dtype=torch.int32, device=dev)
        aliases.append(ne.ne_build_neg_alias(deg_host[lo:hi], lo, table))
    torch.cuda.synchronize()
    log(f"tables + {grid} alias table(s) ready in {time.time() - t0:.1f}s; "
        f"{torch.cuda.memory_allocated() / 2**30:.1f} GiB allocated")

    total_pairs = n_batches * B
    lrs = [np.float32(wl.linear_decay_lr(0.025, i * B, total_pairs)) for i in range(n_batches)]
    pairs = bp.pairs
    pairs_host = None
    if args.pinned_pairs:
        pairs_host = pairs.cpu().pin_memory()
        staging = torch.empty((3, B, 2), dtype=torch.int32, device=dev)

    def bucket_runs(first, last):
        """Batches [first, last) as runs: consecutive batches of one (src-block, ctx-block) bucket."""
        runs, i = [], first
        while i < last:
            s, n, bi, bj = sched[i]
            k = i + 1
            while k < last and sched[k][2:] == (bi, bj) and sched[k][0] == sched[k - 1][0] + B:
                k += 1
            runs.append((i, k, s, bj))
            i = k
        return runs

    def run(first, last):
        """Batches [first, last).  The exact step goes to the library as one ne_train_runs call: the runs of
        consecutive batches of one (src-block, ctx-block) bucket, in the order of the schedule, so that the
        id-only work of every batch but the first rides in the kernels of the batch before it.  --per-run makes
        one ne_train_block call per bucket run, --per-batch one ne_train_batch call per batch."""
        i = first
        while N and i < last:          # shared-negative mode: one call per batch
            s, n, _, bj = sched[i]
            ne.ne_train_batch_shared(tables, aliases[bj], pairs[s:s + n], N, float(lrs[i]), 5.0 / N, i, workspace)
            i += 1
        if args.mode == "async" and i < last:
            for (a, b, s, bj) in bucket_runs(i, last):
                ne.ne_train_block_async(tables, aliases[bj], pairs[s:s + (b - a) * B], B, K, lrs[a:b], a * B)
            return
        if i >= last:
            return
        if args.per_batch:
            for j in range(i, last):
                s, n, _, bj = sched[j]
                ne.ne_train_batch(tables, aliases[bj], pairs[s:s + n], K, float(lrs[j]), j * B)
        elif pairs_host is not None:
            for (a, b, s, bj) in bucket_runs(i, last):
                ne.ne_train_block_pinned(tables, aliases[bj], pairs_host[s:s + (b - a) * B], B, K, lrs[a:b], a * B, staging)
        elif args.per_run:
            for (a, b, s, bj) in bucket_runs(i, last):
                ne.ne_train_block(tables, aliases[bj], pairs[s:s + (b - a) * B], B, K, lrs[a:b], a * B)
        else:
            ne.ne_train_runs(tables, [(aliases[bj], pairs[s:s + (b - a) * B], a * B) for (a, b, s, bj) in bucket_runs(i, last)],
                             B, K, lrs[i:last])

    # args.repeats times: tables initialised again, warm-up, then the timed steps; the median repeat is reported
    samples = []
    for rep in range(args.repeats):
        if rep > 0:
            tables = fresh_tables()
        torch.cuda.synchronize()
        run(0, args.warmup)
        torch.cuda.synchronize()
        ne.ne_profile_enable(tables, 4, args.steps // 4 + 2)
        t_start = time.perf_counter()
        run(args.warmup, n_batches)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t_start
        kern_ms, kern_n = ne.ne_profile_read(tables)
        ne.ne_profile_enable(tables, 0, 0)
        samples.append((elapsed, kern_ms / max(kern_n, 1), kern_n))
        log(f"repeat {rep}: {args.steps * B / elapsed / 1e6:.1f} M pairs/s, {elapsed / args.steps * 1e6:.1f} us/step, "
            f"dominant kernel {kern_ms / max(kern_n, 1) * 1e3:.1f} us")
    samples.sort()
    elapsed, avg_kernel_ms, kern_n = samples[len(samples) // 2]

    pairs_per_s = args.steps * B / elapsed
    copy_GBps = copy_ceiling(dev)
    if N:
        # two gathered rows per pair and the N shared rows per batch, read and written once; ids
        bpp = 2 * (2 * B + N) * 4 * d / B + 8
        flops = 2 * 2.0 * B * N * d          # S and dX products of the scores kernel
        step_flops = 3 * 2.0 * B * N * d     # all three dense products of a step
        achieved = flops / (avg_kernel_ms * 1e-3) / 1e12 if kern_n else None
        step_achieved = step_flops * pairs_per_s / B / 1e12
        roofline = {"bound": "mfma", "kernel": "scores_kernel", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": (achieved / MFMA_BF16_PEAK_TFLOPS) if achieved else None,
                    "traffic": traffic_bytes_per_launch("scores_kernel", name),
                    "flops_per_launch": flops, "avg_kernel_ms": avg_kernel_ms, "kernel_samples": kern_n,
                    "step_achieved": step_achieved, "step_frac": step_achieved / MFMA_BF16_PEAK_TFLOPS,
                    "step_hbm_GBps": pairs_per_s * bpp / 1e9, "step_hbm_frac": pairs_per_s * bpp / 1e9 / HBM_PEAK_GBS}
        call = "ne_train_batch_shared per step"
    else:
        bpp = algorithmic_bytes_per_pair(d, K)
        kernel = "train_kernel"
        achieved = (bpp * B) / (avg_kernel_ms * 1e-3) / 1e9 if kern_n else None
        step_achieved = pairs_per_s * bpp / 1e9
        roofline = {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": (achieved / HBM_PEAK_GBS) if achieved else None,
                    "traffic": traffic_bytes_per_launch(kernel, name) if args.mode == "sync" else None, "bytes_per_launch": bpp * B,
                    "avg_kernel_ms": avg_kernel_ms, "kernel_samples": kern_n,
                    # the whole step (every launch of a batch) on algorithmic bytes: the headline fraction
                    "step_achieved": step_achieved, "step_frac": step_achieved / HBM_PEAK_GBS,
                    "copy_ceiling_GBps": copy_GBps, "step_frac_of_copy_ceiling": step_achieved / copy_GBps}
        call = "ne_train_runs, one call per timed region"
        if args.per_run:
            call = "ne_train_block per bucket run"
        if args.per_batch:
            call = "ne_train_batch per step"
        if pairs_host is not None:
            call = "ne_train_block_pinned per bucket run (pairs prefetched from pinned host memory inside the launches)"
        if args.mode == "async":
            call = "ne_train_block_async per bucket run (per-sample mode, not the exact step)"
    result = {
        "metric": "positive edge samples/sec on 1 MI355X + achieved HBM GB/s vs peak",
        "value": pairs_per_s,
        "unit": "pairs/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "repeats": args.repeats,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if N else "f32",
        "data": "synthetic",
        "config": {"workload": name, "nodes": V, "dim": d, "negatives": N if N else K, "batch": B,
                   "block_grid": f"{grid}x{grid}", "call": call, "end_to_end_GBps": pairs_per_s * bpp / 1e9,
                   "pairs_per_s_of_each_repeat": [args.steps * B / e for e, _, _ in samples]},
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, deg_host, bp, sched, args.cpu_batches)
    print(json.dumps(result), flush=True)


def copy_ceiling(dev) -> float:
    """GB/s (read + write) of a plain 1 GiB device-to-device copy: the practical ceiling beside the datasheet peak."""
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
    dst = torch.empty_like(src)
    dst.copy_(src)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(10):
        dst.copy_(src)
    stop.record()
    torch.cuda.synchronize()
    return 10 * 2 * src.numel() * 4 / (start.elapsed_time(stop) * 1e-3) / 1e9


def walks_scenario(args, dev):
    """Walk workloads trained from the walks themselves (ne_train_walks: 4 bytes per walk entry, the source
    row of an entry gathered once for its window of samples) next to the same batches expanded to pairs
    (ne_train_block: 8 bytes per sample).  Batches are whole walks, i.e. walk-ordered, not shuffled."""
    name = args.workload
    w = WORKLOADS[name]
    if w.get("shared_negatives"):
        print("bench.py: --walks does not apply to the shared-negative workload", file=sys.stderr)
        sys.exit(2)
    V, d, K, B, seed = w["V"], w["d"], w["K"], w["B"], w["seed"]
    L, win = w["walk"] if w["walk"] is not None else w.get("walk_shape", (80, 5))
    per_walk = sum(L - j for j in range(1, win + 1))
    wpb = max(1, B // per_walk)                       # walks per batch: as many whole walks as fit into B samples
    n_batches = args.steps + args.warmup
    if w["walk"] is not None:
        gdev = "cpu" if V <= 100_000 else dev
        g = wl.build_graph(V, wl.rmat_edges(V, w["edges"], seed, w["abc"], device=gdev))
        starts = torch.nonzero(g.degree > 0).reshape(-1)
        gen = torch.Generator(device=starts.device).manual_seed(seed)
        starts = starts[torch.randint(0, starts.numel(), (n_batches * wpb,), generator=gen, device=starts.device)]
        walks = wl.random_walks(g, starts, L, seed).to(torch.int32).to(dev).contiguous()
        degree = g.degree.to(dev)
        del g
    else:
        # Graphs too large to walk here (configs 3, 4): stand-in walks whose entries are drawn like the
        # endpoints of R-MAT edges (a walk visits nodes in proportion to their degree), inside one block of
        # the table grid, negatives from that block.  Same row-access statistics, no graph structure.
        V = V // w["grid"]
        degree = wl.rmat_degrees(V, w["edges"] // w["grid"] ** 2, seed, w["abc"], device=dev)
        walks = (wl.rmat_pairs(w["V"], n_batches * wpb * L // 2 + 1, seed, w["abc"], device=dev).reshape(-1)[: n_batches * wpb * L]
                 % V).to(torch.int32).reshape(n_batches * wpb, L).contiguous()
    # the same samples as pairs, in the order of the walks (entry, then offset)
    parts = [torch.stack([walks[:, :-j], walks[:, j:]], dim=2) for j in range(1, win + 1)]      # [n][L-j][2]
    per_entry = torch.full((walks.shape[0], L, win, 2), -1, dtype=torch.int32, device=dev)
    for j, part in enumerate(parts, start=1):
        per_entry[:, :L - j, j - 1, :] = part
    pairs = per_entry.reshape(walks.shape[0], L * win, 2)
    pairs = pairs[pairs[:, :, 0] >= 0].reshape(walks.shape[0] * per_walk, 2).contiguous()
    Bp = wpb * per_walk
    R = 1 + win * (K + 1)
    max_B = max(Bp, -(-(wpb * L * R) // (K + 2)))
    results = {}
    for mode in ("walks", "pairs"):
        vertex = torch.empty((V, d), dtype=torch.float32, device=dev)
        context = torch.empty((V, d), dtype=torch.float32, device=dev)
        ws = torch.empty(ne.ne_workspace_bytes(d, max_B, K), dtype=torch.uint8, device=dev)
        tables = ne.ne_create_tables(vertex, context, seed, init=True, max_batch=max_B, max_negatives=K, workspace=ws)
        apply_tuning(args, tables)
        at = torch.empty((V, 2), dtype=torch.int32, device=dev)
        alias = ne.ne_build_neg_alias(degree.clamp(max=2**32 - 1).cpu().numpy().astype(np.uint32), 0, at)
        lrs = [np.float32(wl.linear_decay_lr(0.025, i * Bp, n_batches * Bp)) for i in range(n_batches)]

        def run(first, last):
            if mode == "walks":
                ne.ne_train_walks(tables, alias, walks[first * wpb:last * wpb], wpb, win, K, lrs[first:last], first * wpb * L * win)
            else:
                ne.ne_train_block(tables, alias, pairs[first * Bp:last * Bp], Bp, K, lrs[first:last], first * Bp)

        torch.cuda.synchronize()
        run(0, args.warmup)
        torch.cuda.synchronize()
        ne.ne_profile_enable(tables, 4, args.steps // 4 + 2)
        t0 = time.perf_counter()
        run(args.warmup, n_batches)
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        kern_ms, kern_n = ne.ne_profile_read(tables)
        results[mode] = {"pairs_per_s": args.steps * Bp / el, "ms_per_step": el / args.steps * 1e3,
                         "train_kernel_ms": kern_ms / max(kern_n, 1),
                         "sample_bytes_per_step": wpb * L * 4 if mode == "walks" else Bp * 8}
        log(f"walks scenario, {mode}: {results[mode]['pairs_per_s'] / 1e6:.1f} M samples/s, "
            f"{results[mode]['ms_per_step']:.4f} ms/batch, train kernel {results[mode]['train_kernel_ms'] * 1e3:.1f} us")
        del tables, vertex, context, ws
    print(json.dumps({"scenario": "on-device augmentation", "workload": name, "walk_len": L, "window": win,
                      "walks_per_batch": wpb, "samples_per_batch": Bp, "steps": args.steps, "warmup": args.warmup,
                      "ne_train_walks": results["walks"], "ne_train_block_same_batches": results["pairs"]}), flush=True)


def subparts_scenario(args, dev):
    """One source block of config 3 (25 M vertex rows, 12.8 GB) kept in pinned host memory and streamed
    through three device buffers in k sub-parts (Sec. III-B), the context block resident.  Reports the
    streamed rate next to the same work with the block resident and to the copies alone."""
    from paper_2005_13789_amd.subparts import SubpartTrainer
    k = args.subparts
    w = WORKLOADS["c3"]
    d, K, B, seed = w["d"], w["K"], w["B"], w["seed"]
    rows = w["V"] // w["grid"]                     # one block: 25 M rows; ids folded into it
    batches_per_part = max(1, args.steps // k)
    n_pairs = batches_per_part * k * B
    t0 = time.time()
    degree = wl.rmat_degrees(rows, w["edges"] // w["grid"] ** 2, seed, w["abc"], device=dev)
    pairs = wl.rmat_pairs(w["V"], n_pairs, seed, w["abc"], device=dev) % rows        # stand-in: fold into the block
    log(f"subparts: inputs generated in {time.time() - t0:.1f}s")
    context = torch.empty((rows, d), dtype=torch.float32, device=dev)
    vertex = torch.empty((rows, d), dtype=torch.float32, device=dev)
    ws = torch.empty(ne.ne_workspace_bytes(d, B, K), dtype=torch.uint8, device=dev)
    tables = ne.ne_create_tables(vertex, context, seed, init=True, max_batch=B, max_negatives=K, workspace=ws)
    at = torch.empty((rows, 2), dtype=torch.int32, device=dev)
    alias = ne.ne_build_neg_alias(degree.clamp(max=2**32 - 1).cpu().numpy().astype(np.uint32), 0, at)
    host = torch.empty((rows, d), dtype=torch.float32, pin_memory=True)
    host.copy_(vertex)
    tr = SubpartTrainer(tables, host, 0, k)
    part = tr.subpart_of(pairs[:, 0])
    order = torch.argsort(part, stable=True)
    pairs = pairs[order].contiguous()
    counts = torch.bincount(part, minlength=k).cpu().tolist()
    groups, lrs, bases, off = [], [], [], 0
    for s_ in range(k):
        g = pairs[off:off + (counts[s_] // B) * B]          # whole batches only
        groups.append(g)
        lrs.append([0.025] * max(1, g.shape[0] // B))
        bases.append(off)
        off += counts[s_]
    total = sum(g.shape[0] for g in groups)
    torch.cuda.synchronize()

    def timed(fn):
        torch.cuda.synchronize()
        t = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        return time.perf_counter() - t

    def resident():
        ne.ne_set_vertex_window(tables, vertex, 0)
        for s_ in range(k):
            ne.ne_train_block(tables, alias, groups[s_], B, K, lrs[s_], bases[s_])

    def copies_only():
        empty = [g[:0] for g in groups]
        tr.run(alias, empty, B, K, lrs, bases)

    resident()                                   # warm-up
    t_res = timed(resident)
    t_copy = timed(copies_only)
    t_stream = timed(lambda: tr.run(alias, groups, B, K, lrs, bases))
    bpp = algorithmic_bytes_per_pair(d, K)
    print(json.dumps({
        "metric": "positive edge samples/sec on 1 MI355X + achieved HBM GB/s vs peak", "value": total / t_stream,
        "unit": "pairs/s", "n_gpus": 1, "steps": total // B, "warmup": total // B, "ms_per_step": t_stream / (total // B) * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"c3 source block streamed in {k} sub-parts", "block_rows": rows, "dim": d, "negatives": K,
                   "batch": B, "pairs": total, "resident_pairs_per_s": total / t_res, "copies_only_s": t_copy,
                   "streamed_s": t_stream, "resident_s": t_res,
                   "host_link_GBps": 2 * rows * d * 4 / t_copy / 1e9,
                   "end_to_end_GBps": total / t_stream * bpp / 1e9},
        "roofline": None}), flush=True)


def cpu_baseline(w, deg_host, bp, sched, n_cpu_batches):
    """The CPU oracle as it stands, timed on this host on a bounded sample of the same workload."""
    import oracle
    V, d, K, B, seed = w["V"], w["d"], w["K"], w["B"], w["seed"]
    fold = min(V, 1_000_000)          # host tables of the 100 M-node cases do not fit: fold ids mod 1 M
    X, C = oracle.init_tables(fold, d, seed)
    if V == fold:
        deg_fold = deg_host
    else:
        acc = np.zeros(fold, dtype=np.uint64)
        np.add.at(acc, np.arange(V, dtype=np.int64) % fold, deg_host)
        deg_fold = np.minimum(acc, 2**32 - 1).astype(np.uint32)
    thr, alias, _ = oracle.build_alias(deg_fold)

    def batch(i):
        s, n, _, _ = sched[i % len(sched)]
        p = bp.pairs[s:s + n].cpu().numpy()
        return np.ascontiguousarray(p % fold if V != fold else p, dtype=np.int32)

    N = w.get("shared_negatives", 0)

    def run(i, p):
        if N:
            negs = oracle.sample_shared_negatives(seed, i, N, thr, alias, 0)
            oracle.train_batch_shared(X, C, p, negs, 0.025, 5.0 / N, bf16_inputs=True)
        else:
            neg = oracle.sample_negatives(seed, i * B, p.shape[0], K, thr, alias, 0)
            oracle.train_batch(X, C, p, neg, 0.025)

    p0 = batch(0)
    t0 = time.perf_counter()
    run(0, p0)
    first = time.perf_counter() - t0
    if n_cpu_batches <= 0:               # size the one-thread sample to about 10 s of oracle work
        n_cpu_batches = int(max(1, min(256, 10.0 / max(first, 1e-3))))
    batches = [batch(i) for i in range(1, n_cpu_batches + 1)]
    t0 = time.perf_counter()
    done = 0
    for i, p in enumerate(batches, start=1):
        run(i, p)
        done += p.shape[0]
    dt = time.perf_counter() - t0
    sample = f"{n_cpu_batches} batches of {B} pairs"
    if V != fold:
        sample += f" on a row-folded replica (ids mod {fold})"
    one = {"value": done / dt, "unit": "pairs/s", "cores": 1, "kind": "oracle", "sample": sample,
           "seconds": dt, "host_cpus": os.cpu_count()}
    if N:
        return one                       # the shared-negative oracle has no threaded form
    # the same step shared out over the host cores this job may use (per-thread fp64 sums, added in thread order)
    threads = max(1, min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16"))))
    negs = [oracle.sample_negatives(seed, i * B, p.shape[0], K, thr, alias, 0) for i, p in enumerate(batches, start=1)]
    oracle.train_batch_threads(X, C, batches[0], negs[0], 0.025, threads)     # untimed: the threads' pools get their pages
    t0 = time.perf_counter()
    oracle.train_batch_threads(X, C, batches[0], negs[0], 0.025, threads)
    one_pass = (time.perf_counter() - t0) * len(batches)
    reps = int(max(1, min(32, 10.0 / max(one_pass, 1e-3))))                   # about 10 s in all
    t0 = time.perf_counter()
    done_mt = 0
    for _ in range(reps):
        for p, neg in zip(batches, negs):
            oracle.train_batch_threads(X, C, p, neg, 0.025, threads)
            done_mt += p.shape[0]
    dt_mt = time.perf_counter() - t0
    return {"value": done_mt / dt_mt, "unit": "pairs/s", "cores": threads, "kind": "oracle",
            "sample": f"{reps} x {sample}, pairs shared out over {threads} threads (oracle_train_batch_threads; negatives drawn beforehand)",
            "seconds": dt_mt, "host_cpus": os.cpu_count(), "one_thread": one}


if __name__ == "__main__":
    main()
