"""MI355X-native tree decode attention for speculative Tree-of-Thought search.

The package is a thin binding over libspex_tree.so (hand-written HIP for gfx950).
Importing it loads the library and fails if it has not been built.
"""

from .binding import (BF16, F32, FP8_E4M3, NO_NODE, SpexError, SpexTree, spex_tree_append_step,
                      spex_tree_create, spex_tree_decode_attention, spex_tree_destroy,
                      spex_tree_fork, spex_tree_prune)

__all__ = ["SpexTree", "SpexError", "NO_NODE", "F32", "BF16", "FP8_E4M3", "spex_tree_create",
           "spex_tree_destroy", "spex_tree_fork", "spex_tree_append_step", "spex_tree_prune",
           "spex_tree_decode_attention"]
