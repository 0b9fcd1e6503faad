"""Glue between torch input tensors and the numpy oracle -- TEST INFRASTRUCTURE.

Converts the tensors a trace replay hands over (float32, bfloat16, uint8 e4m3
codes; any device) into the raw arrays OracleTree decodes itself.
"""

from __future__ import annotations

import numpy as np
import torch

from .tree_attention import OracleTree, decode_bf16


def raw_array(t: torch.Tensor) -> np.ndarray:
    """float32 -> float32 array, bfloat16 -> uint16 bit patterns, uint8 -> uint8."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype in (torch.float32, torch.float64, torch.uint8):
        return t.numpy()
    raise TypeError(t.dtype)


def queries_fp64(q: torch.Tensor) -> np.ndarray:
    a = raw_array(q)
    return decode_bf16(a) if a.dtype == np.uint16 else a.astype(np.float64)


class OracleSink:
    """Replay target that feeds an OracleTree."""

    def __init__(self, num_q_heads, num_kv_heads, head_dim, kv_dtype, page_size=16):
        self.tree = OracleTree(num_q_heads, num_kv_heads, head_dim, kv_dtype, scale_block=page_size)

    @classmethod
    def for_workload(cls, wl):
        return cls(wl.num_q_heads, wl.num_kv_heads, wl.head_dim, wl.kv_dtype, wl.page_size)

    def fork(self, parent, n):
        return self.tree.fork(parent, n)

    def prune(self, node):
        self.tree.prune(node)

    def append(self, node, k, v, k_scales=None, v_scales=None, n_tokens=None):
        if k is None:
            self.tree.append(node, None, None, n_tokens=n_tokens)
            return
        ks = None if k_scales is None else raw_array(k_scales)
        vs = None if v_scales is None else raw_array(v_scales)
        self.tree.append(node, raw_array(k), raw_array(v), ks, vs)

    def append_quantised(self, node, k, v, k_scales=None, v_scales=None):
        """bf16 tensors into an fp8 oracle tree (the library's quantising append)."""
        ks = None if k_scales is None else raw_array(k_scales)
        vs = None if v_scales is None else raw_array(v_scales)
        self.tree.append_quantised(node, raw_array(k), raw_array(v), ks, vs)
