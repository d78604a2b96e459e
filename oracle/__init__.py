"""ctypes front end of the plain-C CHESS oracle (``chess_oracle.c``).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg import this package.  It shares nothing with
the HIP library: the C file is compiled here with gcc into ``oracle/liboracle.so``
and every array crosses as a numpy buffer.

The functions mirror the C ones; see the header of ``chess_oracle.c`` for the
passages of the paper each follows (Sec. 3.1 Eq. 1-2, Sec. 3.2 Eq. 4 and the
cascade of Alg. 1, and plain softmax attention over the listed pages).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "chess_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

PLAN_BUDGET, PLAN_RATIO, PLAN_FLAT = 0, 1, 2
PROBE_QUERY, PROBE_ANCHOR = 0, 1         # what units are scored against: the query sum, or the Eq. 3 key anchor
SUMMARY_F32, SUMMARY_BF16 = 0, 1         # storage type of the summary vectors
CUT_COUNT, CUT_THRESHOLD = 0, 1          # a level keeps exactly k units / every unit scoring >= the k-th (Alg. 1's S >= tau)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math: fp64 sums must stay in source order)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


class _Geom(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_q_heads", "n_kv_heads", "head_dim", "page_size", "pages_per_chunk", "chunks_per_grid", "max_pages",
                 "summary_dtype")]


class _Plan(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("plan", "sink_pages", "window_pages", "budget_pages", "budget_bp", "over_chunk", "over_grid",
                 "rho_g_bp", "rho_c_bp", "rho_p_bp", "probe", "cut_rule")]


@dataclass(frozen=True)
class Geometry:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    page_size: int
    pages_per_chunk: int
    chunks_per_grid: int
    max_pages: int
    summary_dtype: int = 0          # SUMMARY_F32 | SUMMARY_BF16: how a summary vector is stored (the arrays stay float32)

    @property
    def max_chunks(self) -> int:
        return -(-self.max_pages // self.pages_per_chunk)

    @property
    def max_grids(self) -> int:
        return -(-self.max_chunks // self.chunks_per_grid)

    def _c(self) -> _Geom:
        return _Geom(self.n_q_heads, self.n_kv_heads, self.head_dim, self.page_size, self.pages_per_chunk,
                     self.chunks_per_grid, self.max_pages, self.summary_dtype)


@dataclass(frozen=True)
class Plan:
    plan: int = PLAN_BUDGET
    sink_pages: int = 1
    window_pages: int = 4
    budget_pages: int = 0
    budget_bp: int = 100
    over_chunk: int = 10
    over_grid: int = 5
    rho_g_bp: int = 10000
    rho_c_bp: int = 10000
    rho_p_bp: int = 10000
    probe: int = PROBE_QUERY
    cut_rule: int = CUT_COUNT
    budget_per_seq: "tuple | None" = None    # per-sequence page budgets (an entry > 0 replaces the plan's budget)

    def _c(self) -> _Plan:
        return _Plan(self.plan, self.sink_pages, self.window_pages, self.budget_pages, self.budget_bp,
                     self.over_chunk, self.over_grid, self.rho_g_bp, self.rho_c_bp, self.rho_p_bp, self.probe,
                     self.cut_rule)

    def _per_seq(self, batch: int):
        if self.budget_per_seq is None:
            return None
        a = np.ascontiguousarray(np.asarray(self.budget_per_seq, dtype=np.int32))
        assert a.shape == (batch,)
        return a


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_select.restype = ctypes.c_int
        _lib.oracle_select_shared.restype = ctypes.c_int
    return _lib


def _p(a, ctype):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctype))


def _u16(a: np.ndarray) -> np.ndarray:
    """bf16 payloads travel as their raw 16-bit patterns."""
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def summarize(k_pool, block_table, seq_lens, geom: Geometry):
    """Eq. 1-2.  Returns (page_vec, chunk_vec, grid_vec), fp32, rows past each sequence's counts are 0."""
    k_pool, bt, sl = _u16(k_pool), _i32(block_table), _i32(seq_lens)
    batch = sl.shape[0]
    assert bt.shape == (batch, geom.max_pages)
    shp = (batch, geom.n_kv_heads)
    pv = np.zeros(shp + (geom.max_pages, geom.head_dim), np.float32)
    cv = np.zeros(shp + (geom.max_chunks, geom.head_dim), np.float32)
    gv = np.zeros(shp + (geom.max_grids, geom.head_dim), np.float32)
    g = geom._c()
    _load().oracle_summarize(_p(k_pool, ctypes.c_uint16), _p(bt, ctypes.c_int32), _p(sl, ctypes.c_int32),
                             ctypes.c_int32(batch), ctypes.byref(g), _p(pv, ctypes.c_float),
                             _p(cv, ctypes.c_float), _p(gv, ctypes.c_float))
    return pv, cv, gv


def scores(q, page_vec, chunk_vec, grid_vec, seq_lens, geom: Geometry, plan: "Plan | None" = None):
    """Eq. 4 for every unit of every level, fp64; rows past a sequence's counts are NaN.  The probe is the
    plan's (Eq. 3 anchor over its window, or the query sum); no plan = the query sum."""
    q, sl = _u16(q), _i32(seq_lens)
    batch = sl.shape[0]
    shp = (batch, geom.n_kv_heads)
    ps = np.full(shp + (geom.max_pages,), np.nan)
    cs = np.full(shp + (geom.max_chunks,), np.nan)
    gs = np.full(shp + (geom.max_grids,), np.nan)
    g = geom._c()
    pl = plan._c() if plan is not None else None
    _load().oracle_scores(_p(q, ctypes.c_uint16), _p(page_vec, ctypes.c_float), _p(chunk_vec, ctypes.c_float),
                          _p(grid_vec, ctypes.c_float), _p(sl, ctypes.c_int32), ctypes.c_int32(batch),
                          ctypes.byref(g), ctypes.byref(pl) if pl is not None else None,
                          _p(ps, ctypes.c_double), _p(cs, ctypes.c_double), _p(gs, ctypes.c_double))
    return ps, cs, gs


def select(q, page_vec, chunk_vec, grid_vec, seq_lens, geom: Geometry, plan: Plan, max_sel: int, detail=False):
    """Cascade + union with safety pages.  Returns (page_ids [b,H_kv,max_sel] padded -1, n_selected [b,H_kv]);
    with detail=True also (kept_grid, kept_chunk, counts[k_g,k_c,k_p])."""
    q, sl = _u16(q), _i32(seq_lens)
    batch = sl.shape[0]
    shp = (batch, geom.n_kv_heads)
    ids = np.empty(shp + (max_sel,), np.int32)
    nsel = np.zeros(shp, np.int32)
    kg = np.zeros(shp + (geom.max_grids,), np.uint8)
    kc = np.zeros(shp + (geom.max_chunks,), np.uint8)
    cnt = np.zeros(shp + (3,), np.int32)
    g, p = geom._c(), plan._c()
    per = plan._per_seq(batch)
    rc = _load().oracle_select(_p(q, ctypes.c_uint16), _p(page_vec, ctypes.c_float), _p(chunk_vec, ctypes.c_float),
                               _p(grid_vec, ctypes.c_float), _p(sl, ctypes.c_int32), ctypes.c_int32(batch),
                               ctypes.byref(g), ctypes.byref(p), _p(per, ctypes.c_int32), ctypes.c_int32(max_sel),
                               _p(ids, ctypes.c_int32), _p(nsel, ctypes.c_int32),
                               _p(kg, ctypes.c_uint8), _p(kc, ctypes.c_uint8), _p(cnt, ctypes.c_int32))
    if rc != 0:
        raise ValueError("oracle_select: a row needs more than max_sel page ids")
    return (ids, nsel, kg, kc, cnt) if detail else (ids, nsel)


def anchor(page_vec, seq_lens, geom: Geometry, window_pages: int):
    """Eq. 3: the key anchor of every (sequence, KV head), fp32 [b, H_kv, d]."""
    sl = _i32(seq_lens)
    batch = sl.shape[0]
    out = np.zeros((batch, geom.n_kv_heads, geom.head_dim), np.float32)
    g = geom._c()
    _load().oracle_anchor(_p(np.ascontiguousarray(page_vec), ctypes.c_float), _p(sl, ctypes.c_int32),
                          ctypes.c_int32(batch), ctypes.byref(g), ctypes.c_int32(window_pages), _p(out, ctypes.c_float))
    return out


def select_shared(probes, page_vecs, chunk_vecs, grid_vecs, seq_lens, geom: Geometry, plan: Plan, max_sel: int,
                  detail=False):
    """The cascade under the model-wide scope of Eq. 1: lists of per-layer arrays (probes fp32 [b,H_kv,d] and the
    three summary levels); a unit's score is the sum over layers and KV heads of the per-head dots.  Returns
    (page_ids [b,max_sel] padded -1, n_selected [b]); with detail=True also counts [b,3] = k_g, k_c, k_p."""
    sl = _i32(seq_lens)
    batch, n_layers = sl.shape[0], len(probes)
    assert len(page_vecs) == len(chunk_vecs) == len(grid_vecs) == n_layers

    def table(arrs):
        keep = [np.ascontiguousarray(a, dtype=np.float32) for a in arrs]
        ptrs = (ctypes.POINTER(ctypes.c_float) * n_layers)(*[_p(a, ctypes.c_float) for a in keep])
        return keep, ptrs

    kp, pp = table(probes)
    k1, p1 = table(page_vecs)
    k2, p2 = table(chunk_vecs)
    k3, p3 = table(grid_vecs)
    ids = np.empty((batch, max_sel), np.int32)
    nsel = np.zeros((batch,), np.int32)
    cnt = np.zeros((batch, 3), np.int32)
    g, p = geom._c(), plan._c()
    per = plan._per_seq(batch)
    rc = _load().oracle_select_shared(ctypes.c_int32(n_layers), pp, p1, p2, p3, _p(sl, ctypes.c_int32),
                                      ctypes.c_int32(batch), ctypes.byref(g), ctypes.byref(p), _p(per, ctypes.c_int32),
                                      ctypes.c_int32(max_sel),
                                      _p(ids, ctypes.c_int32), _p(nsel, ctypes.c_int32), _p(cnt, ctypes.c_int32))
    del kp, k1, k2, k3
    if rc != 0:
        raise ValueError("oracle_select_shared: a sequence needs more than max_sel page ids")
    return (ids, nsel, cnt) if detail else (ids, nsel)


def attend(q, k_pool, v_pool, block_table, seq_lens, geom: Geometry, page_ids=None, n_selected=None,
           sm_scale=None, weights_head=None):
    """Softmax attention over the listed pages (all pages if page_ids is None).  Returns out fp32 [b,H_q,d];
    with weights_head=hq also the normalised softmax weights of batch row 0, q head hq."""
    q, k_pool, v_pool = _u16(q), _u16(k_pool), _u16(v_pool)
    bt, sl = _i32(block_table), _i32(seq_lens)
    batch = sl.shape[0]
    if sm_scale is None:
        sm_scale = 1.0 / float(np.sqrt(geom.head_dim))
    out = np.zeros((batch, geom.n_q_heads, geom.head_dim), np.float32)
    max_sel = 0
    if page_ids is not None:
        page_ids, n_selected = _i32(page_ids), _i32(n_selected)
        max_sel = page_ids.shape[-1]
    wts = None
    if weights_head is not None:
        wts = np.zeros(geom.max_pages * geom.page_size + 8, np.float64)
    g = geom._c()
    _load().oracle_attend(_p(q, ctypes.c_uint16), _p(k_pool, ctypes.c_uint16), _p(v_pool, ctypes.c_uint16),
                          _p(bt, ctypes.c_int32), _p(sl, ctypes.c_int32),
                          _p(page_ids, ctypes.c_int32), _p(n_selected, ctypes.c_int32), ctypes.c_int32(max_sel),
                          ctypes.c_int32(batch), ctypes.byref(g), ctypes.c_double(sm_scale),
                          _p(out, ctypes.c_float), _p(wts, ctypes.c_double),
                          ctypes.c_int32(0 if weights_head is None else weights_head))
    return out if weights_head is None else (out, wts)


def entropy(logits_bits, vocab=None):
    """Sec. 3.3: entropy (nats) of softmax(logits) per row; logits as bf16 bit patterns [batch, stride]."""
    z = _u16(logits_bits)
    batch, stride = z.shape
    vocab = stride if vocab is None else vocab
    out = np.zeros((batch,), np.float64)
    _load().oracle_entropy(_p(z, ctypes.c_uint16), ctypes.c_int32(batch), ctypes.c_int32(vocab), ctypes.c_int64(stride),
                           _p(out, ctypes.c_double))
    return out


def page_trigger(H, tau_h: float, tau_v: float):
    """Sec. 3.3 over the steps of one generated page: (mean entropy, variance of the entropy, fire)."""
    h = np.ascontiguousarray(H, dtype=np.float32)
    mean, var, fire = ctypes.c_double(), ctypes.c_double(), ctypes.c_int32()
    _load().oracle_page_trigger(_p(h, ctypes.c_float), ctypes.c_int32(h.shape[0]), ctypes.c_double(tau_h), ctypes.c_double(tau_v),
                                ctypes.byref(mean), ctypes.byref(var), ctypes.byref(fire))
    return mean.value, var.value, bool(fire.value)
