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
    assert L.ne_create_tables(None, 10, 8, fake, fake, 0, 0, None) == ne.NE_ERR_ARG
    assert L.ne_create_tables(ctypes.byref(out), 0, 8, fake, fake, 0, 0, None) == ne.NE_ERR_ARG
    assert L.ne_create_tables(ctypes.byref(out), 10, 6, fake, fake, 0, 0, None) == ne.NE_ERR_ARG
    assert L.ne_create_tables(ctypes.byref(out), 10, 2048, fake, fake, 0, 0, None) == ne.NE_ERR_ARG
    assert L.ne_create_tables(ctypes.byref(out), 2**31, 8, fake, fake, 0, 0, None) == ne.NE_ERR_ARG
    assert L.ne_create_tables(ctypes.byref(out), 10, 8, None, fake, 0, 0, None) == ne.NE_ERR_ARG
    assert L.ne_create_tables(ctypes.byref(out), 10, 8, ctypes.c_void_p(0x1004), fake, 0, 0, None) == ne.NE_ERR_ARG
    assert b"aligned" in L.ne_last_error()
    # bind-only (init = 0) enqueues nothing, so it works without a GPU
    assert L.ne_create_tables(ctypes.byref(out), 10, 8, fake, fake, 7, 0, None) == ne.NE_OK
    tables = out.value
    assert L.ne_train_batch(None, None, fake, 1, 0, 0.1, 0, fake, 1 << 20, None, None) == ne.NE_ERR_ARG
    assert L.ne_train_batch(tables, None, fake, -1, 0, 0.1, 0, fake, 1 << 20, None, None) == ne.NE_ERR_ARG
    assert L.ne_train_batch(tables, None, fake, 1, 64, 0.1, 0, fake, 1 << 20, None, None) == ne.NE_ERR_ARG
    assert L.ne_train_batch(tables, None, fake, 1, 5, 0.1, 0, fake, 1 << 20, None, None) == ne.NE_ERR_ARG
    assert L.ne_train_batch(tables, None, None, 1, 0, 0.1, 0, fake, 1 << 20, None, None) == ne.NE_ERR_ARG
    assert L.ne_train_batch(tables, None, fake, 1, 0, float("nan"), 0, fake, 1 << 20, None, None) == ne.NE_ERR_ARG
    assert L.ne_train_batch(tables, None, fake, 1, 0, 0.1, 0, fake, 8, None, None) == ne.NE_ERR_ARG
    assert b"staging" in L.ne_last_error()
    assert L.ne_train_batch(tables, None, fake, 0, 0, 0.1, 0, None, 0, None, None) == ne.NE_OK   # B = 0
    assert L.ne_eval_loss(tables, None, fake, 1, 0, 0, None, None, None) == ne.NE_ERR_ARG
    assert L.ne_eval_loss(tables, None, fake, 0, 0, 0, fake, None, None) == ne.NE_OK
    assert L.ne_build_neg_alias(ctypes.byref(out), None, 4, 0, fake, None) == ne.NE_ERR_ARG
    deg = (ctypes.c_uint32 * 4)(0, 0, 0, 0)
    assert L.ne_build_neg_alias(ctypes.byref(out), deg, 4, 0, fake, None) == ne.NE_ERR_ARG
    assert b"zero" in L.ne_last_error()
    assert L.ne_build_neg_alias(ctypes.byref(out), deg, 0, 0, fake, None) == ne.NE_ERR_ARG
    assert L.ne_build_neg_alias(ctypes.byref(out), deg, 4, -1, fake, None) == ne.NE_ERR_ARG
    L.ne_destroy_tables(tables)


def test_staging_bytes():
    assert ne.ne_staging_bytes(4096, 128, 5) >= 4096 * (2 * 128 * 4 + 6 * 4 + 5 * 4)
    assert ne.ne_staging_bytes(4096, 130, 5) == 0
    assert ne.ne_staging_bytes(-1, 128, 5) == 0
    assert ne.ne_staging_bytes(10, 128, 64) == 0
    assert ne.ne_staging_bytes(0, 128, 5) > 0
