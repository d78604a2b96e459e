"""ctypes binding of ``libchess.so``: argument marshalling only.

Every method of :class:`Chess` maps one-to-one onto the C entry point of the same name in
``include/chess.h``; tensors are passed as raw device pointers and the launch goes onto torch's
current HIP stream.  There is no fallback: if the library has not been built, loading fails."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

PLAN_BUDGET, PLAN_RATIO, PLAN_FLAT = 0, 1, 2
PROBE_QUERY, PROBE_ANCHOR = 0, 1
CUT_COUNT, CUT_THRESHOLD = 0, 1
SUMMARY_F32, SUMMARY_BF16 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libchess.so")
_lib = None

EXPORTS = ["chess_create", "chess_destroy", "chess_summary_bytes", "chess_summary_layout", "chess_workspace_bytes", "chess_workspace_init",
           "chess_summarize", "chess_summarize_tail", "chess_summarize_recent", "chess_append_kv", "chess_select", "chess_anchor", "chess_select_shared", "chess_entropy", "chess_trigger_update", "chess_monitor_step", "chess_extend_window", "chess_reuse_step", "chess_sparse_decode", "chess_sparse_decode_static", "chess_dense_decode", "chess_decode_step",
           "chess_debug_force_splits", "chess_debug_force_cluster", "chess_debug_force_schedule", "chess_debug_force_general_cut", "chess_debug_set_poll_limit", "chess_workspace_error", "chess_strerror", "chess_version"]


class ChessError(RuntimeError):
    pass


class _CConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_q_heads", "n_kv_heads", "head_dim", "page_size", "pages_per_chunk", "chunks_per_grid",
                 "max_batch", "max_pages_per_seq", "max_selected_pages")] + [("sm_scale", ctypes.c_float),
                                                                              ("summary_dtype", ctypes.c_int32),
                                                                              ("shared_device", ctypes.c_int32)]


class _CPlan(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("plan", "sink_pages", "window_pages", "budget_pages", "budget_bp", "over_chunk", "over_grid",
                 "rho_g_bp", "rho_c_bp", "rho_p_bp", "probe", "cut_rule")] + [("budget_per_seq", ctypes.c_void_p)]


@dataclass(frozen=True)
class Config:
    n_q_heads: int
    n_kv_heads: int
    page_size: int
    max_batch: int
    max_pages_per_seq: int
    max_selected_pages: int
    pages_per_chunk: int = 8
    chunks_per_grid: int = 8
    head_dim: int = 128
    sm_scale: float = 0.0
    summary_dtype: int = SUMMARY_F32
    shared_device: bool = False


@dataclass(frozen=True)
class SelectPlan:
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
    budget_per_seq: object = None      # device int32 tensor [batch] or None (the caller keeps it alive)

    def _c(self) -> _CPlan:
        per = None if self.budget_per_seq is None else ctypes.c_void_p(self.budget_per_seq.data_ptr())
        return _CPlan(self.plan, self.sink_pages, self.window_pages, self.budget_pages, self.budget_bp,
                      self.over_chunk, self.over_grid, self.rho_g_bp, self.rho_c_bp, self.rho_p_bp, self.probe,
                      self.cut_rule, per)


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load the built library; raises if it is missing (build it with ``__graft_entry__.build()``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ChessError(f"{_LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i32p = ctypes.c_void_p, ctypes.c_void_p
        lib.chess_create.argtypes = [ctypes.POINTER(_CConfig), ctypes.POINTER(vp)]
        lib.chess_destroy.argtypes = [vp]
        lib.chess_destroy.restype = None
        lib.chess_summary_bytes.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t)]
        lib.chess_summary_layout.argtypes = [vp] + [ctypes.POINTER(ctypes.c_size_t)] * 3
        lib.chess_workspace_bytes.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t)]
        lib.chess_summarize.argtypes = [vp, vp, i32p, i32p, ctypes.c_int32, i32p, vp, vp]
        lib.chess_summarize_tail.argtypes = [vp, vp, i32p, i32p, ctypes.c_int32, vp, vp]
        lib.chess_summarize_recent.argtypes = [vp, vp, i32p, i32p, ctypes.c_int32, ctypes.c_int32, vp, vp]
        lib.chess_workspace_init.argtypes = [vp, vp, vp]
        lib.chess_select.argtypes = [vp, vp, vp, i32p, ctypes.c_int32, ctypes.POINTER(_CPlan), i32p, i32p, vp, vp]
        lib.chess_entropy.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, vp, vp, vp]
        lib.chess_monitor_step.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_double,
                                           ctypes.c_double, vp, vp, i32p, i32p, vp, vp, vp]
        lib.chess_trigger_update.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_double, ctypes.c_double, vp, i32p, i32p, vp, vp]
        lib.chess_reuse_step.argtypes = [vp, vp, vp, vp, vp, vp, i32p, i32p, i32p, i32p, ctypes.c_int32, vp, vp, vp]
        lib.chess_extend_window.argtypes = [vp, i32p, ctypes.c_int32, i32p, i32p, vp]
        lib.chess_append_kv.argtypes = [vp, vp, vp, vp, vp, i32p, i32p, ctypes.c_int32, i32p, i32p, vp]
        lib.chess_anchor.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int32, i32p, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(vp), vp]
        lib.chess_select_shared.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.c_int32, i32p, ctypes.c_int32,
                                            ctypes.POINTER(_CPlan), i32p, i32p, vp, vp]
        lib.chess_sparse_decode.argtypes = [vp, vp, vp, vp, i32p, i32p, i32p, i32p, ctypes.c_int32, vp, vp, vp]
        lib.chess_sparse_decode_static.argtypes = [vp, vp, vp, vp, i32p, i32p, i32p, i32p, ctypes.c_int32, vp, vp]
        lib.chess_dense_decode.argtypes = [vp, vp, vp, vp, i32p, i32p, ctypes.c_int32, vp, vp, vp]
        lib.chess_decode_step.argtypes = [vp, vp, vp, vp, i32p, i32p, vp, ctypes.c_int32, ctypes.c_int32, vp, i32p, i32p, vp, vp, vp]
        lib.chess_debug_force_splits.argtypes = [vp, ctypes.c_int32, ctypes.c_int32]
        lib.chess_debug_force_cluster.argtypes = [vp, ctypes.c_int32]
        lib.chess_debug_force_general_cut.argtypes = [vp, ctypes.c_int32]
        lib.chess_debug_force_schedule.argtypes = [vp, ctypes.c_int32]
        lib.chess_debug_set_poll_limit.argtypes = [vp, ctypes.c_int32]
        lib.chess_workspace_error.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_int32), vp]
        lib.chess_strerror.argtypes = [ctypes.c_int]
        lib.chess_strerror.restype = ctypes.c_char_p
        lib.chess_version.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class Chess:
    """One configured instance of the library (one layer's shapes).  Methods launch asynchronously on the
    current torch stream and return nothing; outputs are the tensors passed in."""

    def __init__(self, cfg: Config):
        self.lib = load_library()
        self.cfg = cfg
        c = _CConfig(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.page_size, cfg.pages_per_chunk,
                     cfg.chunks_per_grid, cfg.max_batch, cfg.max_pages_per_seq, cfg.max_selected_pages, cfg.sm_scale,
                     cfg.summary_dtype, int(bool(cfg.shared_device)))
        h = ctypes.c_void_p()
        self._check(self.lib.chess_create(ctypes.byref(c), ctypes.byref(h)))
        self._h = h
        n = ctypes.c_size_t()
        self._check(self.lib.chess_summary_bytes(h, ctypes.byref(n)))
        self.summary_bytes = n.value
        self._check(self.lib.chess_workspace_bytes(h, ctypes.byref(n)))
        self.workspace_bytes = n.value
        a, b, c3 = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
        self._check(self.lib.chess_summary_layout(h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c3)))
        self.summary_offsets = (a.value, b.value, c3.value)

    def close(self):
        if getattr(self, "_h", None):
            self.lib.chess_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != 0:
            raise ChessError(f"libchess error {rc}: {self.lib.chess_strerror(rc).decode()}")

    # ---- buffers the caller owns (torch is only the allocator here)
    def new_summaries(self, device="cuda") -> torch.Tensor:
        return torch.zeros(self.summary_bytes, dtype=torch.uint8, device=device)

    def new_workspace(self, device="cuda") -> torch.Tensor:
        ws = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=device)
        self._check(self.lib.chess_workspace_init(self._h, _ptr(ws), _stream()))
        return ws

    def summary_views(self, summaries: torch.Tensor):
        """(pages, chunks, grids) views [max_batch, H_kv, units, d] of a summaries buffer, fp32 or bf16 by the
        configuration's summary_dtype."""
        c = self.cfg
        mc = -(-c.max_pages_per_seq // c.pages_per_chunk)
        mg = -(-mc // c.chunks_per_grid)
        dt, size = (torch.bfloat16, 2) if c.summary_dtype == SUMMARY_BF16 else (torch.float32, 4)
        out = []
        for off, units in zip(self.summary_offsets, (c.max_pages_per_seq, mc, mg)):
            n = c.max_batch * c.n_kv_heads * units * c.head_dim
            out.append(summaries[off:off + size * n].view(dt).view(c.max_batch, c.n_kv_heads, units, c.head_dim))
        return tuple(out)

    # ---- the C entry points
    def summarize(self, k_pool, block_table, seq_lens, summaries, from_page=None):
        self._check(self.lib.chess_summarize(self._h, _ptr(k_pool), _ptr(block_table), _ptr(seq_lens),
                                             seq_lens.shape[0], _ptr(from_page), _ptr(summaries), _stream()))

    def summarize_tail(self, k_pool, block_table, seq_lens, summaries):
        self._check(self.lib.chess_summarize_tail(self._h, _ptr(k_pool), _ptr(block_table), _ptr(seq_lens),
                                                  seq_lens.shape[0], _ptr(summaries), _stream()))

    def summarize_recent(self, k_pool, block_table, seq_lens, recent_pages: int, summaries):
        self._check(self.lib.chess_summarize_recent(self._h, _ptr(k_pool), _ptr(block_table), _ptr(seq_lens),
                                                    seq_lens.shape[0], recent_pages, _ptr(summaries), _stream()))

    def select(self, q, summaries, seq_lens, plan: SelectPlan, page_ids, n_selected, workspace):
        p = plan._c()
        self._check(self.lib.chess_select(self._h, _ptr(q), _ptr(summaries), _ptr(seq_lens), seq_lens.shape[0],
                                          ctypes.byref(p), _ptr(page_ids), _ptr(n_selected), _ptr(workspace), _stream()))

    def entropy(self, logits, entropy, workspace, vocab=None):
        self._check(self.lib.chess_entropy(self._h, _ptr(logits), logits.shape[0], logits.shape[1] if vocab is None else vocab,
                                           logits.stride(0), _ptr(entropy), _ptr(workspace), _stream()))

    def monitor_step(self, logits, page_steps: int, tau_entropy: float, tau_variance: float, entropy, history, count, fire,
                     workspace, stats=None, vocab=None):
        self._check(self.lib.chess_monitor_step(self._h, _ptr(logits), logits.shape[0],
                                                logits.shape[1] if vocab is None else vocab, logits.stride(0), page_steps,
                                                tau_entropy, tau_variance, _ptr(entropy), _ptr(history), _ptr(count),
                                                _ptr(fire), _ptr(stats), _ptr(workspace), _stream()))

    def trigger_update(self, entropy, page_steps: int, tau_entropy: float, tau_variance: float, history, count, fire,
                       stats=None):
        self._check(self.lib.chess_trigger_update(self._h, _ptr(entropy), entropy.shape[0], page_steps, tau_entropy,
                                                  tau_variance, _ptr(history), _ptr(count), _ptr(fire), _ptr(stats), _stream()))

    def reuse_step(self, q, k_new, v_new, k_pool, v_pool, block_table, seq_lens, page_ids, n_selected, out, workspace):
        self._check(self.lib.chess_reuse_step(self._h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_pool), _ptr(v_pool),
                                              _ptr(block_table), _ptr(seq_lens), _ptr(page_ids), _ptr(n_selected),
                                              seq_lens.shape[0], _ptr(out), _ptr(workspace), _stream()))

    def extend_window(self, seq_lens, page_ids, n_selected):
        self._check(self.lib.chess_extend_window(self._h, _ptr(seq_lens), seq_lens.shape[0], _ptr(page_ids), _ptr(n_selected),
                                                 _stream()))

    def append_kv(self, k_new, v_new, k_pool, v_pool, block_table, seq_lens, page_ids=None, n_selected=None):
        self._check(self.lib.chess_append_kv(self._h, _ptr(k_new), _ptr(v_new), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                                             _ptr(seq_lens), seq_lens.shape[0], _ptr(page_ids), _ptr(n_selected), _stream()))

    def anchor(self, summaries, seq_lens, window_pages: int, anchors):
        """summaries / anchors: one device tensor each, or sequences of per-layer tensors (one launch)."""
        if isinstance(summaries, torch.Tensor):
            summaries, anchors = [summaries], [anchors]
        n = len(summaries)
        assert len(anchors) == n
        st = (ctypes.c_void_p * n)(*[t.data_ptr() for t in summaries])
        at = (ctypes.c_void_p * n)(*[t.data_ptr() for t in anchors])
        self._check(self.lib.chess_anchor(self._h, st, n, _ptr(seq_lens), seq_lens.shape[0], window_pages, at, _stream()))

    def select_shared(self, probes, summaries, seq_lens, plan: SelectPlan, page_ids, n_selected, workspace):
        """probes / summaries: sequences of per-layer device tensors."""
        n = len(probes)
        assert len(summaries) == n
        pt = (ctypes.c_void_p * n)(*[t.data_ptr() for t in probes])
        st = (ctypes.c_void_p * n)(*[t.data_ptr() for t in summaries])
        p = plan._c()
        self._check(self.lib.chess_select_shared(self._h, pt, st, n, _ptr(seq_lens), seq_lens.shape[0], ctypes.byref(p),
                                                 _ptr(page_ids), _ptr(n_selected), _ptr(workspace), _stream()))

    def sparse_decode(self, q, k_pool, v_pool, block_table, seq_lens, page_ids, n_selected, out, workspace):
        self._check(self.lib.chess_sparse_decode(self._h, _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                                                 _ptr(seq_lens), _ptr(page_ids), _ptr(n_selected), seq_lens.shape[0],
                                                 _ptr(out), _ptr(workspace), _stream()))

    def sparse_decode_static(self, q, k_pool, v_pool, block_table, seq_lens, page_ids, n_selected, out):
        self._check(self.lib.chess_sparse_decode_static(self._h, _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                                                        _ptr(seq_lens), _ptr(page_ids), _ptr(n_selected), seq_lens.shape[0],
                                                        _ptr(out), _stream()))

    def dense_decode(self, q, k_pool, v_pool, block_table, seq_lens, out, workspace):
        self._check(self.lib.chess_dense_decode(self._h, _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                                                _ptr(seq_lens), seq_lens.shape[0], _ptr(out), _ptr(workspace), _stream()))

    def decode_step(self, q, k_pool, v_pool, block_table, seq_lens, summaries, plan: SelectPlan, page_ids, n_selected,
                    out, workspace, refresh_tail: bool = False):
        p = plan._c()
        self._check(self.lib.chess_decode_step(self._h, _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                                               _ptr(seq_lens), _ptr(summaries), int(bool(refresh_tail)),
                                               seq_lens.shape[0], ctypes.byref(p),
                                               _ptr(page_ids), _ptr(n_selected), _ptr(out), _ptr(workspace), _stream()))

    def workspace_error(self, workspace) -> int:
        flag = ctypes.c_int32()
        self._check(self.lib.chess_workspace_error(self._h, _ptr(workspace), ctypes.byref(flag), _stream()))
        return flag.value

    def debug_force_cluster(self, cluster: int):
        self._check(self.lib.chess_debug_force_cluster(self._h, cluster))

    def debug_force_schedule(self, schedule: int):
        """0 = automatic, 1 = lazy, 2 = merged."""
        self._check(self.lib.chess_debug_force_schedule(self._h, schedule))

    def debug_force_general_cut(self, on: bool):
        self._check(self.lib.chess_debug_force_general_cut(self._h, int(bool(on))))

    def debug_set_poll_limit(self, polls: int):
        self._check(self.lib.chess_debug_set_poll_limit(self._h, polls))

    def debug_force_splits(self, n_splits: int, waves: int = 4):
        self._check(self.lib.chess_debug_force_splits(self._h, n_splits, waves))
