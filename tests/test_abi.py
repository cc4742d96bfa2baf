"""The C-ABI library loads and exports every function include/ne.h declares; host-side argument
checks return errors without touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2005_13789_amd as ne

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ne.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ne_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree():
    names = declared_functions()
    assert set(names) == set(ne.EXPORTS)
    for required in ("ne_create_tables", "ne_build_neg_alias", "ne_train_batch", "ne_eval_loss"):
        assert required in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(ne.LIB_PATH):
        pytest.fail("libne.so is not built: python -m paper_2005_13789_amd.build")
    L = ctypes.CDLL(ne.LIB_PATH)
    for name in declared_functions():
        assert hasattr(L, name), name


def test_host_side_argument_errors():
    L = ne.lib()
    out = ctypes.c_void_p()
    fake = ctypes.c_void_p(0x1000)      # never dereferenced: every call below fails on the host first

    def create(nodes=10, dim=8, v=fake, c=fake, max_b=0, max_k=0, ws=None, ws_bytes=0, outp=ctypes.byref(out)):
        return L.ne_create_tables(outp, nodes, dim, v, c, 0, 0, max_b, max_k, ws, ws_bytes, None)

    assert create(outp=None) == ne.NE_ERR_ARG
    assert create(nodes=0) == ne.NE_ERR_ARG
    assert create(dim=6) == ne.NE_ERR_ARG
    assert create(dim=2048) == ne.NE_ERR_ARG
    assert create(nodes=2**31) == ne.NE_ERR_ARG
    assert create(v=None) == ne.NE_ERR_ARG
    assert create(v=ctypes.c_void_p(0x1004)) == ne.NE_ERR_ARG
    assert b"aligned" in L.ne_last_error()
    assert create(max_b=16, max_k=5, ws=None) == ne.NE_ERR_ARG           # training without workspace
    assert create(max_b=16, max_k=5, ws=fake, ws_bytes=64) == ne.NE_ERR_ARG   # workspace too small
    assert b"workspace" in L.ne_last_error()
    assert create(max_b=16, max_k=63, ws=fake, ws_bytes=1 << 30) == ne.NE_ERR_ARG
    # bind-only (init = 0, no workspace) enqueues nothing, so it works without a GPU
    assert create() == ne.NE_OK
    tables = out.value
    assert L.ne_train_batch(None, None, fake, 1, 0, 0.1, 0, None, None) == ne.NE_ERR_ARG
    assert L.ne_train_batch(tables, None, fake, -1, 0, 0.1, 0, None, None) == ne.NE_ERR_ARG
    assert L.ne_train_batch(tables, None, fake, 1, 63, 0.1, 0, None, None) == ne.NE_ERR_ARG
    assert L.ne_train_batch(tables, None, fake, 1, 5, 0.1, 0, None, None) == ne.NE_ERR_ARG      # K > 0, no alias
    assert L.ne_train_batch(tables, None, None, 1, 0, 0.1, 0, None, None) == ne.NE_ERR_ARG
    assert L.ne_train_batch(tables, None, fake, 1, 0, float("nan"), 0, None, None) == ne.NE_ERR_ARG
    assert L.ne_train_batch(tables, None, fake, 1, 0, 0.1, 0, None, None) == ne.NE_ERR_STATE    # no workspace
    assert b"workspace" in L.ne_last_error()
    lr = (ctypes.c_float * 2)(0.1, 0.1)
    assert L.ne_train_block(tables, None, fake, 10, 0, 0, lr, 0, None, None) == ne.NE_ERR_ARG       # B = 0
    assert L.ne_train_block(tables, None, fake, -5, 8, 0, lr, 0, None, None) == ne.NE_ERR_ARG
    assert L.ne_train_block(tables, None, fake, 10, 8, 0, None, 0, None, None) == ne.NE_ERR_ARG     # no lr
    assert L.ne_train_block(tables, None, fake, 10, 8, 0, lr, 0, None, None) == ne.NE_ERR_STATE     # no workspace
    assert L.ne_train_block(tables, None, fake, 0, 8, 0, lr, 0, None, None) == ne.NE_OK             # nothing to do
    # runs: (tables, runs, n_runs, B, K, lr, stream)
    one = (ne.NeRun * 1)(ne.NeRun(None, fake.value, 10, 0, None))
    assert L.ne_train_runs(None, one, 1, 8, 0, lr, None) == ne.NE_ERR_ARG
    assert L.ne_train_runs(tables, None, 1, 8, 0, lr, None) == ne.NE_ERR_ARG
    assert L.ne_train_runs(tables, one, -1, 8, 0, lr, None) == ne.NE_ERR_ARG
    assert L.ne_train_runs(tables, one, 1, 0, 0, lr, None) == ne.NE_ERR_ARG             # B = 0
    assert L.ne_train_runs(tables, one, 1, 8, 0, None, None) == ne.NE_ERR_ARG           # no lr
    assert L.ne_train_runs(tables, one, 1, 8, 3, lr, None) == ne.NE_ERR_ARG             # K > 0, no alias
    assert L.ne_train_runs(tables, one, 1, 8, 0, lr, None) == ne.NE_ERR_STATE           # no workspace
    assert L.ne_train_runs(tables, one, 0, 8, 0, lr, None) == ne.NE_OK                  # nothing to do
    assert L.ne_eval_loss(tables, None, fake, 1, 0, 0, None, None, None) == ne.NE_ERR_ARG
    assert L.ne_eval_loss(tables, None, fake, 0, 0, 0, fake, None, None) == ne.NE_OK            # B = 0
    assert L.ne_build_neg_alias(ctypes.byref(out), None, 4, 0, fake, None) == ne.NE_ERR_ARG
    deg = (ctypes.c_uint32 * 4)(0, 0, 0, 0)
    assert L.ne_build_neg_alias(ctypes.byref(out), deg, 4, 0, fake, None) == ne.NE_ERR_ARG
    assert b"zero" in L.ne_last_error()
    assert L.ne_build_neg_alias(ctypes.byref(out), deg, 0, 0, fake, None) == ne.NE_ERR_ARG
    assert L.ne_build_neg_alias(ctypes.byref(out), deg, 4, -1, fake, None) == ne.NE_ERR_ARG
    # walks: (tables, alias, walks, n_walks, walks_per_batch, walk_len, window, K, lr, sample_base, neg_out, stream)
    def walks(tb=tables, al=None, w=fake, n=4, wpb=2, length=10, window=3, K=0, lrs=lr):
        return L.ne_train_walks(tb, al, w, n, wpb, length, window, K, lrs, 0, None, None)

    assert walks(tb=None) == ne.NE_ERR_ARG
    assert walks(K=63) == ne.NE_ERR_ARG
    assert walks(K=5) == ne.NE_ERR_ARG                  # K > 0, no alias
    assert walks(length=1) == ne.NE_ERR_ARG
    assert walks(length=65537) == ne.NE_ERR_ARG
    assert walks(window=0) == ne.NE_ERR_ARG
    assert walks(window=65) == ne.NE_ERR_ARG
    assert b"window" in L.ne_last_error()
    assert walks(n=-1) == ne.NE_ERR_ARG
    assert walks(n=0, w=None) == ne.NE_OK               # nothing to do
    assert walks(w=None) == ne.NE_ERR_ARG
    assert walks(w=ctypes.c_void_p(0x1002)) == ne.NE_ERR_ARG
    assert walks(wpb=0) == ne.NE_ERR_ARG
    assert walks(lrs=None) == ne.NE_ERR_ARG
    assert walks(lrs=(ctypes.c_float * 2)(0.1, float("inf"))) == ne.NE_ERR_ARG
    assert walks() == ne.NE_ERR_STATE                   # no workspace
    # pinned pairs: (tables, alias, pairs_host, n_pairs, B, K, lr, sample_base, staging, neg_out, stream); a NULL
    # host pointer is refused before any HIP call is made
    assert L.ne_train_block_pinned(tables, None, None, 10, 8, 0, lr, 0, fake, None, None) == ne.NE_ERR_ARG
    assert b"pairs_host_pinned" in L.ne_last_error()
    assert L.ne_train_block_pinned(None, None, None, 0, 8, 0, lr, 0, fake, None, None) == ne.NE_ERR_ARG
    assert L.ne_train_block_pinned(tables, None, None, 0, 8, 0, lr, 0, None, None, None) == ne.NE_OK        # no pairs: nothing to do
    # scores: (tables, pairs, n, second_from_context, scores, stream)
    assert L.ne_score_pairs(None, fake, 1, 1, fake, None) == ne.NE_ERR_ARG
    assert L.ne_score_pairs(tables, fake, -1, 1, fake, None) == ne.NE_ERR_ARG
    assert L.ne_score_pairs(tables, None, 1, 1, fake, None) == ne.NE_ERR_ARG
    assert L.ne_score_pairs(tables, ctypes.c_void_p(0x1004), 1, 1, fake, None) == ne.NE_ERR_ARG
    assert L.ne_score_pairs(tables, fake, 1, 1, None, None) == ne.NE_ERR_ARG
    assert L.ne_score_pairs(tables, None, 0, 1, None, None) == ne.NE_OK
    assert L.ne_set_tuning(None, -1, 0) == ne.NE_ERR_ARG
    assert L.ne_set_tuning(tables, -2, 0) == ne.NE_ERR_ARG
    assert L.ne_set_tuning(tables, 9, 0) == ne.NE_ERR_ARG
    assert L.ne_set_tuning(tables, 0, 3) == ne.NE_ERR_ARG
    assert b"sweep_per_thread" in L.ne_last_error()
    assert L.ne_set_tuning(tables, 8, 2) == ne.NE_OK
    assert L.ne_set_tuning(tables, -1, 0) == ne.NE_OK
    assert L.ne_validate_pairs(tables, fake, 1, None, None) == ne.NE_ERR_ARG
    assert L.ne_validate_pairs(tables, fake, -1, fake, None) == ne.NE_ERR_ARG
    assert L.ne_validate_pairs(tables, None, 0, fake, None) == ne.NE_OK
    L.ne_destroy_tables(tables)


def test_workspace_bytes():
    w = ne.ne_workspace_bytes(128, 4096, 5)
    refs = 4096 * 7
    assert w >= 2 * refs * 128 * 4 + 2 * refs * 4
    assert ne.ne_workspace_bytes(130, 4096, 5) == 0
    assert ne.ne_workspace_bytes(128, 0, 5) == 0
    assert ne.ne_workspace_bytes(128, 10, 63) == 0
    assert ne.ne_workspace_bytes(128, ne.NE_MAX_BATCH + 1, 5) == 0
    assert ne.ne_workspace_bytes(128, 8192, 5) > w
