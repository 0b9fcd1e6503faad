"""Seeded synthetic inputs for tree decode attention.

This package produces the *inputs* both the HIP library and the CPU oracle are
fed with: counter-based random K/V/Q values, the fp8 encoding of those values,
and the fork / append / prune traces that shape the five benchmark trees.  It
holds none of the attention arithmetic and imports neither the library binding
nor the oracle.
"""

from .rng import normal_values, hash_key
from .quant import encode_e4m3, quantise_pages
from .trees import (Workload, TreeOp, ValueProfile, tiny_tree, bfs_tot, mcts_skewed,
                    spec_at_scale, tot_with_drafts, step_prefill, random_trace, draft_tree_masks,
                    with_draft_trees, WORKLOADS)
from .replay import replay, gen_queries

__all__ = [
    "normal_values", "hash_key", "encode_e4m3", "quantise_pages", "Workload", "TreeOp", "ValueProfile",
    "tiny_tree", "bfs_tot", "mcts_skewed", "spec_at_scale", "tot_with_drafts", "step_prefill",
    "random_trace", "draft_tree_masks", "with_draft_trees", "WORKLOADS", "replay", "gen_queries",
]
