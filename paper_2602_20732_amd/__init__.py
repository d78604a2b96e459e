"""MI355X-native decode hot path of CHESS (hierarchical KV page selection + block-sparse paged decode).

The product is ``libchess.so`` (hand-written HIP kernels behind the C ABI declared in ``include/chess.h``);
this package is the thin Python binding over it.  PyTorch is used only for device memory and streams."""
from .binding import (PLAN_BUDGET, PLAN_FLAT, PLAN_RATIO, PROBE_ANCHOR, PROBE_QUERY, CUT_COUNT, CUT_THRESHOLD, SUMMARY_F32, SUMMARY_BF16, Chess, ChessError, Config, SelectPlan, library_path,
                      load_library)

__all__ = ["Chess", "ChessError", "Config", "SelectPlan", "PLAN_BUDGET", "PLAN_RATIO", "PLAN_FLAT", "PROBE_QUERY", "PROBE_ANCHOR", "CUT_COUNT", "CUT_THRESHOLD", "SUMMARY_F32", "SUMMARY_BF16", "library_path", "load_library"]
