"""MI355X-native quantised-histogram tree construction (arXiv 1806.11248).

The product is ``libgbt.so`` (hand-written HIP for gfx950 behind a C ABI, see
``include/gbt.h``); this package is its thin ctypes binding.
"""
from .binding import (Context, GbtError, LIB_PATH, OBJECTIVES, Params, SYMBOLS, bits_for, load, make_params,  # noqa: F401
                      new_tree, new_tree_leaves, packed_words)
