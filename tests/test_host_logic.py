"""CPU-side checks of the product's host logic: the C-ABI library loads without a GPU, exports every
symbol ``include/chess.h`` declares, and rejects bad arguments before touching the device."""
from __future__ import annotations

import ctypes
import os
import re

import pytest

import paper_2602_20732_amd as pk
from paper_2602_20732_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pk.library_path()):
        from paper_2602_20732_amd.build import build
        build()
    return pk.load_library()


def declared_symbols():
    """Every function the public header and the test-hook header declare."""
    names = set()
    for header in ("chess.h", "chess_debug.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        found = set(re.findall(r"\b(chess_[a-z_]+)\s*\(", text))
        hooks = {n for n in found if n.startswith("chess_debug_")}
        assert hooks == (found if header == "chess_debug.h" else set()), "test hooks, and only they, belong in chess_debug.h"
        names |= found
    return sorted(names)


def test_library_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names, "binding and header list the same entry points"


def test_version_and_error_strings(lib):
    assert lib.chess_version() == 1
    for code in (0, -1, -2, -3, -4, -99):
        assert lib.chess_strerror(code)


def test_create_rejects_bad_shapes_before_touching_the_device(lib):
    h = ctypes.c_void_p()
    assert lib.chess_create(None, ctypes.byref(h)) == -1
    ok = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, page_size=16, pages_per_chunk=8, chunks_per_grid=8,
              max_batch=1, max_pages_per_seq=2048, max_selected_pages=26, sm_scale=0.0)
    for bad in (dict(head_dim=64), dict(page_size=8), dict(n_kv_heads=5), dict(n_q_heads=8 * 17),
                dict(pages_per_chunk=0), dict(pages_per_chunk=32, chunks_per_grid=16), dict(max_batch=0),
                dict(max_selected_pages=4096), dict(sm_scale=-1.0), dict(sm_scale=float("nan"))):
        c = binding._CConfig(**{**ok, **bad})
        assert lib.chess_create(ctypes.byref(c), ctypes.byref(h)) == -1, bad
        assert not h.value


def test_null_context_is_rejected(lib):
    n = ctypes.c_size_t()
    assert lib.chess_summary_bytes(None, ctypes.byref(n)) == -1
    assert lib.chess_workspace_bytes(None, ctypes.byref(n)) == -1
    assert lib.chess_workspace_init(None, None, None) == -1
    assert lib.chess_select(None, None, None, None, 1, None, None, None, None, None) == -1
    assert lib.chess_dense_decode(None, None, None, None, None, None, 1, None, None, None) == -1
    lib.chess_destroy(None)
