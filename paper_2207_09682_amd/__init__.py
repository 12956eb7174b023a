"""MI355X-native hot path of quantized GBDT training (arxiv 2207.09682).

The package is a thin binding over the in-tree HIP library `libqgbdt.so`
(C ABI in include/qgbdt.h).  It has no CPU implementation.
"""
from .binding import (Context, QgbdtError, Tree, ROUND_NEAREST, ROUND_STOCHASTIC, ROWS_AUTO, ROWS_IDS,
                      ROWS_IDS_GH, ROWS_ORDERED, EXPORTS, LIB_PATH, load_library, unpack_hist, unpack_splits)

__all__ = ["Context", "QgbdtError", "Tree", "ROUND_NEAREST", "ROUND_STOCHASTIC", "ROWS_AUTO", "ROWS_IDS", "ROWS_IDS_GH",
           "ROWS_ORDERED", "EXPORTS", "LIB_PATH",
           "load_library", "unpack_hist", "unpack_splits"]
