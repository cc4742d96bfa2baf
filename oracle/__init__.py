"""ctypes front end of the CPU oracle (``ne_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  Nothing under the product package imports it, and it imports
nothing from the product package.  All arrays are host numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ne_oracle.c")
_SO = os.path.join(_HERE, "libne_oracle.so")

_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc.  No fast-math, no FMA contraction: plain IEEE fp64."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-Wextra", "-pthread", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build(force=False)
    _lib = _bind(ctypes.CDLL(_SO))
    return _lib


def _bind(lib):
    """Declare the C signatures on a loaded copy of the oracle library."""
    c = ctypes
    p = c.c_void_p
    lib.oracle_philox4x32_10.argtypes = [p, p, p]
    lib.oracle_philox4x32_10.restype = None
    lib.oracle_init_tables.argtypes = [c.c_int64, c.c_int32, c.c_uint64, p, p]
    lib.oracle_init_tables.restype = None
    lib.oracle_build_alias.argtypes = [p, c.c_int64, p, p, p]
    lib.oracle_build_alias.restype = c.c_int
    lib.oracle_sample_negatives.argtypes = [c.c_uint64, c.c_uint64, c.c_int64, c.c_int32, p, p,
                                            c.c_int64, c.c_int32, p]
    lib.oracle_sample_negatives.restype = None
    lib.oracle_sample_shared_negatives.argtypes = [c.c_uint64, c.c_uint64, c.c_int32, p, p,
                                                   c.c_int64, c.c_int32, p]
    lib.oracle_sample_shared_negatives.restype = None
    lib.oracle_train_batch.argtypes = [p, p, c.c_int64, c.c_int32, p, c.c_int64, c.c_int32,
                                       c.c_float, p]
    lib.oracle_train_batch.restype = c.c_int
    lib.oracle_train_batch_threads.argtypes = [p, p, c.c_int64, c.c_int32, p, c.c_int64, c.c_int32,
                                               c.c_float, p, c.c_int32]
    lib.oracle_train_batch_threads.restype = c.c_int
    lib.oracle_train_batch_shared.argtypes = [p, p, c.c_int64, c.c_int32, p, c.c_int64, p, c.c_int32, c.c_float,
                                              c.c_float, c.c_int32, c.POINTER(c.c_double)]
    lib.oracle_train_batch_shared.restype = c.c_int
    lib.oracle_train_sequential.argtypes = [p, p, c.c_int64, c.c_int32, p, c.c_int64, c.c_int32, c.c_float, p]
    lib.oracle_train_sequential.restype = c.c_int
    lib.oracle_score_pairs.argtypes = [p, p, c.c_int32, p, c.c_int64, c.c_int32, p]
    lib.oracle_score_pairs.restype = None
    lib.oracle_walk_pairs.argtypes = [p, c.c_int64, c.c_int32, c.c_int32, p, p]
    lib.oracle_walk_pairs.restype = c.c_int64
    lib.oracle_eval_loss.argtypes = [p, p, c.c_int64, c.c_int32, p, c.c_int64, c.c_int32, p]
    lib.oracle_eval_loss.restype = c.c_double
    return lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _chk(a, dtype, name):
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: need a C-contiguous numpy array of {np.dtype(dtype)}")
    return a


def philox4x32_10(ctr, key) -> np.ndarray:
    """Four 32-bit outputs of Philox4x32-10 for counter (c0..c3) and key (k0, k1)."""
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    assert ctr.shape == (4,) and key.shape == (2,)
    out = np.empty(4, dtype=np.uint32)
    _load().oracle_philox4x32_10(_ptr(ctr), _ptr(key), _ptr(out))
    return out


def init_tables(num_nodes: int, dim: int, seed: int):
    """(vertex, context) fp32 tables: vertex ~ U(-0.5/dim, 0.5/dim), context = 0."""
    X = np.empty((num_nodes, dim), dtype=np.float32)
    C = np.empty((num_nodes, dim), dtype=np.float32)
    _load().oracle_init_tables(num_nodes, dim, seed, _ptr(X), _ptr(C))
    return X, C


def build_alias(degree: np.ndarray):
    """Alias table for P(i) ~ degree_i^0.75.  Returns (thr_q uint32[n], alias uint32[n], prob f64[n])."""
    degree = _chk(np.ascontiguousarray(degree, dtype=np.uint32), np.uint32, "degree")
    n = degree.shape[0]
    thr = np.empty(n, dtype=np.uint32)
    alias = np.empty(n, dtype=np.uint32)
    prob = np.empty(n, dtype=np.float64)
    rc = _load().oracle_build_alias(_ptr(degree), n, _ptr(thr), _ptr(alias), _ptr(prob))
    if rc != 0:
        raise ValueError(f"oracle_build_alias failed ({rc}): empty input or all degrees zero")
    return thr, alias, prob


def sample_negatives(seed: int, sample_base: int, B: int, K: int, thr: np.ndarray,
                     alias: np.ndarray, base: int = 0) -> np.ndarray:
    """int32[B][K] negative ids for samples sample_base .. sample_base+B-1."""
    _chk(thr, np.uint32, "thr")
    _chk(alias, np.uint32, "alias")
    out = np.empty((B, K), dtype=np.int32)
    _load().oracle_sample_negatives(seed, sample_base, B, K, _ptr(thr), _ptr(alias), thr.shape[0],
                                    base, _ptr(out))
    return out


def sample_shared_negatives(seed: int, batch_index: int, N: int, thr: np.ndarray, alias: np.ndarray,
                            base: int = 0) -> np.ndarray:
    """int32[N] negative ids shared by every pair of batch `batch_index`."""
    _chk(thr, np.uint32, "thr")
    _chk(alias, np.uint32, "alias")
    out = np.empty(N, dtype=np.int32)
    _load().oracle_sample_shared_negatives(seed, batch_index, N, _ptr(thr), _ptr(alias),
                                           thr.shape[0], base, _ptr(out))
    return out


def train_batch(X: np.ndarray, C: np.ndarray, pairs: np.ndarray, neg: np.ndarray, lr: float) -> None:
    """One minibatch-synchronous SGNS step, in place on X and C (fp32 [V][d])."""
    _chk(X, np.float32, "X")
    _chk(C, np.float32, "C")
    _chk(pairs, np.int32, "pairs")
    _chk(neg, np.int32, "neg")
    V, d = X.shape
    B = pairs.shape[0]
    assert C.shape == X.shape and pairs.shape == (B, 2)
    K = neg.shape[1] if B > 0 else (neg.shape[1] if neg.ndim == 2 else 0)
    assert neg.shape == (B, K)
    rc = _load().oracle_train_batch(_ptr(X), _ptr(C), V, d, _ptr(pairs), B, K, np.float32(lr),
                                    _ptr(neg))
    if rc != 0:
        raise ValueError(f"oracle_train_batch failed ({rc})")


def train_batch_threads(X: np.ndarray, C: np.ndarray, pairs: np.ndarray, neg: np.ndarray, lr: float,
                        threads: int) -> None:
    """train_batch with the pairs shared out over host threads (per-thread fp64 sums added in thread order);
    exists for timing the oracle on all cores."""
    _chk(X, np.float32, "X")
    _chk(C, np.float32, "C")
    _chk(pairs, np.int32, "pairs")
    _chk(neg, np.int32, "neg")
    V, d = X.shape
    B = pairs.shape[0]
    assert C.shape == X.shape and pairs.shape == (B, 2) and neg.ndim == 2 and neg.shape[0] == B
    rc = _load().oracle_train_batch_threads(_ptr(X), _ptr(C), V, d, _ptr(pairs), B, neg.shape[1], np.float32(lr),
                                            _ptr(neg), int(threads))
    if rc != 0:
        raise ValueError(f"oracle_train_batch_threads failed ({rc})")


def eval_loss(X: np.ndarray, C: np.ndarray, pairs: np.ndarray, neg: np.ndarray) -> float:
    """Sum over the batch of -log s(s_0) - sum_k log s(-s_k) at the current tables."""
    _chk(X, np.float32, "X")
    _chk(C, np.float32, "C")
    _chk(pairs, np.int32, "pairs")
    _chk(neg, np.int32, "neg")
    V, d = X.shape
    B = pairs.shape[0]
    K = neg.shape[1]
    assert neg.shape == (B, K)
    return float(_load().oracle_eval_loss(_ptr(X), _ptr(C), V, d, _ptr(pairs), B, K, _ptr(neg)))


def train_batch_shared(X: np.ndarray, C: np.ndarray, pairs: np.ndarray, negs: np.ndarray, lr: float,
                       neg_scale: float, bf16_inputs: bool = True) -> float:
    """Shared-negative step in place on X and C; returns the summed loss at the pre-batch tables.

    Every pair is scored against all N ids of negs (int32[N]); negative terms carry weight neg_scale.
    bf16_inputs rounds the rows and the coefficients of the dense products to bfloat16 first.
    """
    _chk(X, np.float32, "X")
    _chk(C, np.float32, "C")
    _chk(pairs, np.int32, "pairs")
    _chk(negs, np.int32, "negs")
    V, d = X.shape
    B = pairs.shape[0]
    loss = ctypes.c_double()
    rc = _load().oracle_train_batch_shared(_ptr(X), _ptr(C), V, d, _ptr(pairs), B, _ptr(negs), negs.shape[0],
                                           np.float32(lr), np.float32(neg_scale), 1 if bf16_inputs else 0,
                                           ctypes.byref(loss))
    if rc != 0:
        raise ValueError(f"oracle_train_batch_shared failed ({rc})")
    return loss.value


def train_sequential(X: np.ndarray, C: np.ndarray, pairs: np.ndarray, neg: np.ndarray, lr: float) -> None:
    """Per-sample SGD in the order of pairs, in place: each sample sees what the ones before it left."""
    _chk(X, np.float32, "X")
    _chk(C, np.float32, "C")
    _chk(pairs, np.int32, "pairs")
    _chk(neg, np.int32, "neg")
    V, d = X.shape
    B = pairs.shape[0]
    K = neg.shape[1]
    assert neg.shape == (B, K)
    rc = _load().oracle_train_sequential(_ptr(X), _ptr(C), V, d, _ptr(pairs), B, K, np.float32(lr), _ptr(neg))
    if rc != 0:
        raise ValueError(f"oracle_train_sequential failed ({rc})")


def score_pairs(X: np.ndarray, C: np.ndarray, pairs: np.ndarray, second_from_context: bool = True) -> np.ndarray:
    """float64[n]: X[pairs[i,0]] . (C if second_from_context else X)[pairs[i,1]]."""
    _chk(X, np.float32, "X")
    _chk(C, np.float32, "C")
    _chk(pairs, np.int32, "pairs")
    out = np.empty(pairs.shape[0], dtype=np.float64)
    _load().oracle_score_pairs(_ptr(X), _ptr(C), X.shape[1], _ptr(pairs), pairs.shape[0],
                               1 if second_from_context else 0, _ptr(out))
    return out


def walk_pairs(walks: np.ndarray, window: int):
    """Samples of walks int32[n][L] (Algorithm 1, augmentation): (pairs int32[m][2], sample index int64[m])."""
    _chk(walks, np.int32, "walks")
    n, L = walks.shape
    pairs = np.empty((n * L * window, 2), dtype=np.int32)
    sample = np.empty(n * L * window, dtype=np.int64)
    m = _load().oracle_walk_pairs(_ptr(walks), n, L, window, _ptr(pairs), _ptr(sample))
    return np.ascontiguousarray(pairs[:m]), np.ascontiguousarray(sample[:m])
