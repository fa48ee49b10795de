"""The C-ABI library loads and exports every symbol include/evict.h declares; host-only
argument checks return the documented status codes (no GPU work is launched here)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2605_00342_amd as ev

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.skipif(not ev.is_built(), reason="libevict.so not built (run __graft_entry__.build())")


def test_header_symbols_are_exported():
    text = open(os.path.join(ROOT, "include", "evict.h")).read()
    declared = set(re.findall(r"\b(evict_[a-z_]+)\s*\(", text))
    assert declared == set(ev.EXPORTS)
    lib = ev.load()
    for name in declared:
        assert hasattr(lib, name), name
    assert ev.evict_version() >= 1


def test_validate_trees_host():
    off = np.array([0, 4, 7], np.int32)
    par = np.array([-1, 0, 0, 2, -1, 0, 1], np.int32)
    assert ev.evict_validate_trees_host(off, par, 2, 128) == 0
    bad = par.copy(); bad[3] = 3
    assert ev.evict_validate_trees_host(off, bad, 2, 128) == 1
    assert "parent" in ev.evict_last_error()
    bad = par.copy(); bad[4] = 0
    assert ev.evict_validate_trees_host(off, bad, 2, 128) == 1
    assert ev.evict_validate_trees_host(off, par, 2, 3) == 1
    assert ev.evict_validate_trees_host(np.array([0, 0, 7], np.int32), par, 2, 128) == 1


def test_host_side_argument_checks_need_no_gpu():
    lib = ev.load()
    # null pointers and bad sizes are rejected before anything is launched
    assert lib.evict_select_prefix(None, None, None, None, 1, 1, None, 1, None, None, None, None, None, None, None, None) == 1
    assert lib.evict_accept_path(None, None, None, None, None, 1, None, 1, None, None, None) == 1
    assert lib.evict_expert_union(None, None, 1, 1, 1, None, None, None, None, None, None, None) == 1
    one = ctypes.c_void_p(16)
    assert lib.evict_expert_union(None, one, 4, 9, 8, one, one, one, one, one, one, None) == 1      # k > E
    assert lib.evict_expert_union(None, one, 4096, 8, 128, one, one, one, one, one, one, None) == 2  # too large
    assert lib.evict_gather_rows(one, one, 6, one, one, one, 1, 1, None) == 1                       # row_bytes % 4
    d = ev.ModelDesc(ev.EVICT_BF16, 2048, 32, 5, 128, 128, 8, 768, 0, 1e-6, 1e6, 0)
    h = ctypes.c_void_p()
    assert lib.evict_create(ctypes.byref(h), ctypes.byref(d), 32, 1, 2048) == 1                      # Hq % Hkv
    d = ev.ModelDesc(ev.EVICT_BF16, 2048, 32, 4, 96, 128, 8, 768, 0, 1e-6, 1e6, 0)
    assert lib.evict_create(ctypes.byref(h), ctypes.byref(d), 32, 1, 2048) == 2                      # head dim
    assert lib.evict_pack_dense(ev.EVICT_BF16, one, 24, 64, ctypes.c_void_p(32), None) == 2          # rows % 16
    assert ev.evict_packed_bytes(ev.EVICT_BF16, 2048, 768) == 2048 * 768 * 2
    assert lib.evict_destroy(None) == 0
