"""Python binding of libne.so, the MI355X SGNS node-embedding training library.

Argument marshalling only: every function below forwards to the C entry point of the same name
(see include/ne.h).  torch is used for device memory and streams; all arithmetic runs in the HIP
kernels.  Importing the package does not load the library; the first call does, and it raises if
the library has not been built (there is no fallback path).
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libne.so")

NE_OK = 0
NE_ERR_ARG = -1
NE_ERR_STATE = -2
NE_ERR_HIP = -3
NE_ERR_NOMEM = -4
NE_MAX_DIM = 1024
NE_MAX_NEGATIVES = 62
NE_MAX_BATCH = 1 << 22

EXPORTS = (
    "ne_create_tables", "ne_build_neg_alias", "ne_workspace_bytes", "ne_train_batch", "ne_train_block", "ne_train_runs", "ne_train_block_pinned", "ne_train_walks",
    "ne_shared_workspace_bytes", "ne_train_batch_shared", "ne_train_batch_shared_static", "ne_train_batch_async", "ne_train_block_async", "ne_set_vertex_window", "ne_eval_loss",
    "ne_score_pairs", "ne_set_tuning", "ne_validate_pairs", "ne_hash_position", "ne_profile_enable", "ne_profile_read", "ne_destroy_tables", "ne_destroy_alias", "ne_last_error",
)

_lib = None


class NeRun(ctypes.Structure):
    """struct ne_run of include/ne.h."""
    _fields_ = [("alias", ctypes.c_void_p), ("pairs_dev", ctypes.c_void_p), ("n_pairs", ctypes.c_int64),
                ("sample_base", ctypes.c_uint64), ("neg_out_dev", ctypes.c_void_p)]


class NeError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"ne status {status}: {message}")
        self.status = status


def lib() -> ctypes.CDLL:
    """Load libne.so (once).  Raises if it is missing: build it with paper_2005_13789_amd/build.py."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: run `python -m paper_2005_13789_amd.build` (hipcc, gfx950) first")
    L = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp = c.c_void_p
    L.ne_create_tables.argtypes = [c.POINTER(vp), c.c_int64, c.c_int32, vp, vp, c.c_uint64, c.c_int32, c.c_int64,
                                   c.c_int32, vp, c.c_size_t, vp]
    L.ne_create_tables.restype = c.c_int
    L.ne_build_neg_alias.argtypes = [c.POINTER(vp), vp, c.c_int64, c.c_int32, vp, vp]
    L.ne_build_neg_alias.restype = c.c_int
    L.ne_workspace_bytes.argtypes = [c.c_int32, c.c_int64, c.c_int32]
    L.ne_workspace_bytes.restype = c.c_size_t
    L.ne_train_batch.argtypes = [vp, vp, vp, c.c_int64, c.c_int32, c.c_float, c.c_uint64, vp, vp]
    L.ne_train_batch.restype = c.c_int
    L.ne_train_block.argtypes = [vp, vp, vp, c.c_int64, c.c_int64, c.c_int32, c.POINTER(c.c_float), c.c_uint64, vp, vp]
    L.ne_train_block.restype = c.c_int
    L.ne_train_runs.argtypes = [vp, c.POINTER(NeRun), c.c_int64, c.c_int64, c.c_int32, c.POINTER(c.c_float), vp]
    L.ne_train_runs.restype = c.c_int
    L.ne_train_block_pinned.argtypes = [vp, vp, vp, c.c_int64, c.c_int64, c.c_int32, c.POINTER(c.c_float), c.c_uint64, vp,
                                        vp, vp]
    L.ne_train_block_pinned.restype = c.c_int
    L.ne_shared_workspace_bytes.argtypes = [c.c_int32, c.c_int64, c.c_int32]
    L.ne_shared_workspace_bytes.restype = c.c_size_t
    L.ne_train_batch_shared.argtypes = [vp, vp, vp, c.c_int64, c.c_int32, c.c_float, c.c_float, c.c_uint64, vp,
                                        c.c_size_t, vp, vp, vp]
    L.ne_train_batch_shared.restype = c.c_int
    L.ne_train_batch_shared_static.argtypes = [vp, vp, vp, c.c_int64, c.c_int32, c.c_float, c.c_float, c.c_uint64, vp, vp, vp]
    L.ne_train_batch_shared_static.restype = c.c_int
    L.ne_train_batch_async.argtypes = [vp, vp, vp, c.c_int64, c.c_int32, c.c_float, c.c_uint64, vp, vp]
    L.ne_train_batch_async.restype = c.c_int
    L.ne_train_block_async.argtypes = [vp, vp, vp, c.c_int64, c.c_int64, c.c_int32, c.POINTER(c.c_float), c.c_uint64, vp, vp]
    L.ne_train_block_async.restype = c.c_int
    L.ne_set_vertex_window.argtypes = [vp, vp, c.c_int64, c.c_int64]
    L.ne_set_vertex_window.restype = c.c_int
    L.ne_eval_loss.argtypes = [vp, vp, vp, c.c_int64, c.c_int32, c.c_uint64, vp, vp, vp]
    L.ne_eval_loss.restype = c.c_int
    L.ne_train_walks.argtypes = [vp, vp, vp, c.c_int64, c.c_int64, c.c_int32, c.c_int32, c.c_int32, c.POINTER(c.c_float),
                                 c.c_uint64, vp, vp]
    L.ne_train_walks.restype = c.c_int
    L.ne_score_pairs.argtypes = [vp, vp, c.c_int64, c.c_int32, vp, vp]
    L.ne_score_pairs.restype = c.c_int
    L.ne_set_tuning.argtypes = [vp, c.c_int32, c.c_int32]
    L.ne_set_tuning.restype = c.c_int
    L.ne_validate_pairs.argtypes = [vp, vp, c.c_int64, vp, vp]
    L.ne_validate_pairs.restype = c.c_int
    L.ne_hash_position.argtypes = [c.c_uint32, c.c_uint32]
    L.ne_hash_position.restype = c.c_uint32
    L.ne_profile_enable.argtypes = [vp, c.c_int32, c.c_int32]
    L.ne_profile_enable.restype = c.c_int
    L.ne_profile_read.argtypes = [vp, c.POINTER(c.c_double), c.POINTER(c.c_int64)]
    L.ne_profile_read.restype = c.c_int
    L.ne_destroy_tables.argtypes = [vp]
    L.ne_destroy_tables.restype = None
    L.ne_destroy_alias.argtypes = [vp]
    L.ne_destroy_alias.restype = None
    L.ne_last_error.argtypes = []
    L.ne_last_error.restype = c.c_char_p
    _lib = L
    return L


def _check(status: int) -> None:
    if status != NE_OK:
        raise NeError(status, lib().ne_last_error().decode("utf-8", "replace"))


def _stream_ptr(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dev_ptr(t, dtype, name: str) -> int:
    if t is None:
        return 0
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: need a contiguous CUDA tensor of {dtype}")
    return t.data_ptr()


class Tables:
    """Handle from ne_create_tables; keeps the table and workspace tensors alive."""

    def __init__(self, handle: int, vertex: torch.Tensor, context: torch.Tensor, seed: int, workspace):
        self.handle = handle
        self.vertex = vertex
        self.context = context
        self.seed = seed
        self.workspace = workspace
        self.num_nodes, self.dim = vertex.shape

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.ne_destroy_tables(self.handle)
            self.handle = None


class Alias:
    """Handle from ne_build_neg_alias; keeps the device table tensor alive."""

    def __init__(self, handle: int, table: torch.Tensor, n: int, base: int):
        self.handle = handle
        self.table = table
        self.n = n
        self.base = base

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.ne_destroy_alias(self.handle)
            self.handle = None


def ne_workspace_bytes(dim: int, max_batch: int, max_negatives: int) -> int:
    return int(lib().ne_workspace_bytes(dim, max_batch, max_negatives))


def ne_create_tables(vertex: torch.Tensor, context: torch.Tensor, seed: int, init: bool = True,
                     max_batch: int = 0, max_negatives: int = 0, workspace: torch.Tensor | None = None,
                     stream=None) -> Tables:
    """Bind fp32 [num_nodes][dim] CUDA tensors; if init, vertex ~ U(-0.5/dim, 0.5/dim), context = 0.

    workspace: CUDA uint8 tensor of ne_workspace_bytes(dim, max_batch, max_negatives) bytes (needed
    for ne_train_batch; leave None with max_batch = 0 for an evaluate-only handle).
    """
    vp = _dev_ptr(vertex, torch.float32, "vertex")
    cp = _dev_ptr(context, torch.float32, "context")
    if vertex.dim() != 2 or vertex.shape != context.shape:
        raise TypeError("vertex and context must both be [num_nodes][dim]")
    wp = _dev_ptr(workspace, torch.uint8, "workspace")
    out = ctypes.c_void_p()
    _check(lib().ne_create_tables(ctypes.byref(out), vertex.shape[0], vertex.shape[1], vp, cp,
                                  seed & (2**64 - 1), 1 if init else 0, max_batch, max_negatives, wp,
                                  workspace.numel() if workspace is not None else 0, _stream_ptr(stream)))
    return Tables(out.value, vertex, context, seed, workspace)


def ne_build_neg_alias(degree_host, base: int, alias_table: torch.Tensor, stream=None) -> Alias:
    """degree_host: CPU uint32-valued array/tensor [n]; alias_table: CUDA int32 [n][2] to be filled."""
    import numpy as np
    if isinstance(degree_host, torch.Tensor):
        degree_host = degree_host.cpu().numpy()
    deg = np.ascontiguousarray(degree_host, dtype=np.uint32)
    n = int(deg.shape[0])
    ap = _dev_ptr(alias_table, torch.int32, "alias_table")
    if alias_table.numel() < 2 * n:
        raise TypeError("alias_table needs 2*n int32 elements")
    out = ctypes.c_void_p()
    _check(lib().ne_build_neg_alias(ctypes.byref(out), deg.ctypes.data, n, base, ap, _stream_ptr(stream)))
    return Alias(out.value, alias_table, n, base)


def ne_train_batch(tables: Tables, alias: Alias | None, pairs: torch.Tensor, K: int, lr: float,
                   sample_base: int, neg_out: torch.Tensor | None = None, stream=None,
                   B: int | None = None) -> None:
    """One minibatch-synchronous SGNS step on pairs int32 [B][2] (CUDA)."""
    if B is None:
        B = int(pairs.shape[0])
    pp = _dev_ptr(pairs, torch.int32, "pairs")
    np_ = _dev_ptr(neg_out, torch.int32, "neg_out")
    if neg_out is not None and neg_out.numel() < B * K:
        raise TypeError("neg_out needs B*K int32 elements")
    _check(lib().ne_train_batch(tables.handle, alias.handle if alias else None, pp, B, K, lr, sample_base,
                                np_, _stream_ptr(stream)))


def ne_train_block(tables: Tables, alias: Alias | None, pairs: torch.Tensor, B: int, K: int, lrs,
                   sample_base: int, neg_out: torch.Tensor | None = None, stream=None) -> None:
    """All of pairs int32 [n_pairs][2] (CUDA) in consecutive batches of B; lrs: one float per batch."""
    n_pairs = int(pairs.shape[0])
    n_batches = -(-n_pairs // B) if B > 0 else 0
    if len(lrs) < n_batches:
        raise TypeError("lrs needs one learning rate per batch")
    arr = (ctypes.c_float * max(n_batches, 1))(*[float(v) for v in lrs[:n_batches]])
    pp = _dev_ptr(pairs, torch.int32, "pairs")
    np_ = _dev_ptr(neg_out, torch.int32, "neg_out")
    if neg_out is not None and neg_out.numel() < n_pairs * K:
        raise TypeError("neg_out needs n_pairs*K int32 elements")
    _check(lib().ne_train_block(tables.handle, alias.handle if alias else None, pp, n_pairs, B, K, arr, sample_base,
                                np_, _stream_ptr(stream)))


def ne_train_runs(tables: Tables, runs, B: int, K: int, lrs, stream=None) -> None:
    """runs: sequence of (alias, pairs int32 [n][2] CUDA, sample_base) or (alias, pairs, sample_base, neg_out);
    lrs: one float per batch, the runs' batches in order."""
    arr = (NeRun * max(len(runs), 1))()
    n_batches = 0
    for i, run in enumerate(runs):
        alias, pairs, sample_base = run[0], run[1], run[2]
        neg_out = run[3] if len(run) > 3 else None
        n = int(pairs.shape[0])
        if neg_out is not None and neg_out.numel() < n * K:
            raise TypeError("neg_out needs n_pairs*K int32 elements")
        arr[i] = NeRun(alias.handle if alias else None, _dev_ptr(pairs, torch.int32, "pairs") or None, n, sample_base,
                       _dev_ptr(neg_out, torch.int32, "neg_out") or None)
        n_batches += -(-n // B) if B > 0 else 0
    if len(lrs) < n_batches:
        raise TypeError("lrs needs one learning rate per batch")
    lr_arr = (ctypes.c_float * max(n_batches, 1))(*[float(v) for v in lrs[:n_batches]])
    _check(lib().ne_train_runs(tables.handle, arr, len(runs), B, K, lr_arr, _stream_ptr(stream)))


def ne_train_block_pinned(tables: Tables, alias: Alias | None, pairs_host: torch.Tensor, B: int, K: int, lrs,
                          sample_base: int, staging: torch.Tensor, neg_out: torch.Tensor | None = None, stream=None) -> None:
    """ne_train_block on pairs in pinned CPU memory (int32 [n][2]); staging: CUDA int32 [3][B][2]."""
    if not (isinstance(pairs_host, torch.Tensor) and not pairs_host.is_cuda and pairs_host.dtype == torch.int32
            and pairs_host.is_contiguous() and pairs_host.is_pinned()):
        raise TypeError("pairs_host: need a contiguous pinned CPU tensor of torch.int32")
    n_pairs = int(pairs_host.shape[0])
    n_batches = -(-n_pairs // B) if B > 0 else 0
    if len(lrs) < n_batches:
        raise TypeError("lrs needs one learning rate per batch")
    arr = (ctypes.c_float * max(n_batches, 1))(*[float(v) for v in lrs[:n_batches]])
    sp = _dev_ptr(staging, torch.int32, "staging")
    if staging.numel() < 6 * B:
        raise ValueError("staging needs 3*B*2 int32 elements")
    np_ = _dev_ptr(neg_out, torch.int32, "neg_out")
    if neg_out is not None and neg_out.numel() < n_pairs * K:
        raise TypeError("neg_out needs n_pairs*K int32 elements")
    _check(lib().ne_train_block_pinned(tables.handle, alias.handle if alias else None, pairs_host.data_ptr(), n_pairs, B, K,
                                       arr, sample_base, sp, np_, _stream_ptr(stream)))


def ne_train_walks(tables: Tables, alias: Alias | None, walks: torch.Tensor, walks_per_batch: int, window: int, K: int,
                   lrs, sample_base: int, neg_out: torch.Tensor | None = None, stream=None) -> None:
    """All of walks int32 [n_walks][walk_len] (CUDA) in consecutive batches of walks_per_batch walks; lrs: one float
    per batch.  neg_out: int32 [n_walks][walk_len][window][K] or None."""
    n_walks, walk_len = int(walks.shape[0]), int(walks.shape[1])
    n_batches = -(-n_walks // walks_per_batch) if walks_per_batch > 0 else 0
    if len(lrs) < n_batches:
        raise TypeError("lrs needs one learning rate per batch")
    arr = (ctypes.c_float * max(n_batches, 1))(*[float(v) for v in lrs[:n_batches]])
    wp = _dev_ptr(walks, torch.int32, "walks")
    np_ = _dev_ptr(neg_out, torch.int32, "neg_out")
    if neg_out is not None and neg_out.numel() < n_walks * walk_len * window * K:
        raise TypeError("neg_out needs n_walks*walk_len*window*K int32 elements")
    _check(lib().ne_train_walks(tables.handle, alias.handle if alias else None, wp, n_walks, walks_per_batch, walk_len,
                                window, K, arr, sample_base, np_, _stream_ptr(stream)))


def ne_train_batch_async(tables: Tables, alias: Alias | None, pairs: torch.Tensor, K: int, lr: float,
                         sample_base: int, neg_out: torch.Tensor | None = None, stream=None) -> None:
    """Per-sample step on pairs int32 [B][2] (CUDA): no update is lost, but pairs that share a row do not wait
    for each other (shared rows take atomic adds on the table while other pairs may still read them)."""
    B = int(pairs.shape[0])
    pp = _dev_ptr(pairs, torch.int32, "pairs")
    np_ = _dev_ptr(neg_out, torch.int32, "neg_out")
    if neg_out is not None and neg_out.numel() < B * K:
        raise TypeError("neg_out needs B*K int32 elements")
    _check(lib().ne_train_batch_async(tables.handle, alias.handle if alias else None, pp, B, K, lr, sample_base,
                                      np_, _stream_ptr(stream)))


def ne_train_block_async(tables: Tables, alias: Alias | None, pairs: torch.Tensor, B: int, K: int, lrs,
                         sample_base: int, neg_out: torch.Tensor | None = None, stream=None) -> None:
    """ne_train_batch_async on all of pairs int32 [n_pairs][2] (CUDA) in consecutive batches of B; lrs: one float per batch."""
    n_pairs = int(pairs.shape[0])
    n_batches = -(-n_pairs // B) if B > 0 else 0
    if len(lrs) < n_batches:
        raise TypeError("lrs needs one learning rate per batch")
    arr = (ctypes.c_float * max(n_batches, 1))(*[float(v) for v in lrs[:n_batches]])
    pp = _dev_ptr(pairs, torch.int32, "pairs")
    np_ = _dev_ptr(neg_out, torch.int32, "neg_out")
    if neg_out is not None and neg_out.numel() < n_pairs * K:
        raise TypeError("neg_out needs n_pairs*K int32 elements")
    _check(lib().ne_train_block_async(tables.handle, alias.handle if alias else None, pp, n_pairs, B, K, arr, sample_base,
                                      np_, _stream_ptr(stream)))


def ne_set_vertex_window(tables: Tables, window: torch.Tensor, first_row: int) -> None:
    """Vertex rows [first_row, first_row + len(window)) now live in `window` (CUDA fp32 [rows][dim])."""
    wp = _dev_ptr(window, torch.float32, "window")
    if window.dim() != 2 or window.shape[1] != tables.dim:
        raise TypeError("window must be [rows][dim]")
    _check(lib().ne_set_vertex_window(tables.handle, wp, first_row, int(window.shape[0])))
    tables.vertex_window = window      # keep it alive while the handle points at it


def ne_shared_workspace_bytes(dim: int, B: int, N: int) -> int:
    return int(lib().ne_shared_workspace_bytes(dim, B, N))


def ne_train_batch_shared(tables: Tables, alias: Alias, pairs: torch.Tensor, N: int, lr: float, neg_scale: float,
                          batch_index: int, workspace: torch.Tensor, neg_out: torch.Tensor | None = None,
                          loss_sum: torch.Tensor | None = None, stream=None) -> None:
    """Shared-negative step: every pair of pairs int32 [B][2] (CUDA) against the same N negatives."""
    B = int(pairs.shape[0])
    pp = _dev_ptr(pairs, torch.int32, "pairs")
    wp = _dev_ptr(workspace, torch.uint8, "workspace")
    np_ = _dev_ptr(neg_out, torch.int32, "neg_out")
    lp = _dev_ptr(loss_sum, torch.float64, "loss_sum")
    if neg_out is not None and neg_out.numel() < N:
        raise TypeError("neg_out needs N int32 elements")
    _check(lib().ne_train_batch_shared(tables.handle, alias.handle if alias else None, pp, B, N, lr, neg_scale,
                                       batch_index, wp, workspace.numel(), np_, lp, _stream_ptr(stream)))


NE_SHARED_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024


def ne_train_batch_shared_static(tables: Tables, alias: Alias, pairs: torch.Tensor, N: int, lr: float, neg_scale: float,
                                 batch_index: int, neg_out: torch.Tensor | None = None,
                                 loss_sum: torch.Tensor | None = None, stream=None) -> None:
    """ne_train_batch_shared on the library's static per-GPU scratch (no workspace argument, nothing allocated);
    shapes whose workspace exceeds NE_SHARED_STATIC_SCRATCH_BYTES are refused."""
    B = int(pairs.shape[0])
    pp = _dev_ptr(pairs, torch.int32, "pairs")
    np_ = _dev_ptr(neg_out, torch.int32, "neg_out")
    lp = _dev_ptr(loss_sum, torch.float64, "loss_sum")
    if neg_out is not None and neg_out.numel() < N:
        raise TypeError("neg_out needs N int32 elements")
    _check(lib().ne_train_batch_shared_static(tables.handle, alias.handle if alias else None, pp, B, N, lr, neg_scale,
                                              batch_index, np_, lp, _stream_ptr(stream)))


def ne_eval_loss(tables: Tables, alias: Alias | None, pairs: torch.Tensor, K: int, sample_base: int,
                 loss_sum: torch.Tensor, neg_out: torch.Tensor | None = None, stream=None,
                 B: int | None = None) -> None:
    """Adds the batch's summed SGNS loss to loss_sum (CUDA float64 scalar tensor)."""
    if B is None:
        B = int(pairs.shape[0])
    pp = _dev_ptr(pairs, torch.int32, "pairs")
    lp = _dev_ptr(loss_sum, torch.float64, "loss_sum")
    np_ = _dev_ptr(neg_out, torch.int32, "neg_out")
    if neg_out is not None and neg_out.numel() < B * K:
        raise TypeError("neg_out needs B*K int32 elements")
    _check(lib().ne_eval_loss(tables.handle, alias.handle if alias else None, pp, B, K, sample_base, lp, np_,
                              _stream_ptr(stream)))


def ne_score_pairs(tables: Tables, pairs: torch.Tensor, scores: torch.Tensor, second_from_context: bool = True,
                   stream=None) -> None:
    """scores[i] = vertex[pairs[i,0]] . (context if second_from_context else vertex)[pairs[i,1]] (CUDA float32[n])."""
    pp = _dev_ptr(pairs, torch.int32, "pairs")
    sp = _dev_ptr(scores, torch.float32, "scores")
    if scores.numel() < pairs.shape[0]:
        raise ValueError("scores is shorter than pairs")
    _check(lib().ne_score_pairs(tables.handle, pp, int(pairs.shape[0]), 1 if second_from_context else 0, sp,
                                _stream_ptr(stream)))


def ne_set_tuning(tables: Tables, list_cap: int = -1, sweep_per_thread: int = 0) -> None:
    """How the exact step collects the deltas of rows that several references name (list_cap: -1 automatic,
    0 atomics only, up to 8 listed references per row) and how finely the apply kernel sweeps (0 automatic, 2, 4, 8)."""
    _check(lib().ne_set_tuning(tables.handle, list_cap, sweep_per_thread))


def ne_validate_pairs(tables: Tables, pairs: torch.Tensor, bad_count: torch.Tensor, stream=None) -> None:
    """Adds the number of out-of-range ids in pairs to bad_count (CUDA int64 scalar tensor)."""
    pp = _dev_ptr(pairs, torch.int32, "pairs")
    bp = _dev_ptr(bad_count, torch.int64, "bad_count")
    _check(lib().ne_validate_pairs(tables.handle, pp, int(pairs.shape[0]), bp, _stream_ptr(stream)))


def ne_hash_position(key: int, positions: int) -> int:
    """Home position of a row key among `positions` hash positions (host-only debug helper)."""
    return int(lib().ne_hash_position(key & 0xFFFFFFFF, positions))


def ne_profile_enable(tables: Tables, every_n: int, max_samples: int = 4096) -> None:
    """Record HIP events around the train kernel of every n-th ne_train_batch call (0 = off)."""
    _check(lib().ne_profile_enable(tables.handle, every_n, max_samples))


def ne_profile_read(tables: Tables):
    """(sum of the sampled train-kernel durations in ms, number of samples); resets the samples."""
    total = ctypes.c_double()
    n = ctypes.c_int64()
    _check(lib().ne_profile_read(tables.handle, ctypes.byref(total), ctypes.byref(n)))
    return total.value, n.value


def ne_last_error() -> str:
    return lib().ne_last_error().decode("utf-8", "replace")
