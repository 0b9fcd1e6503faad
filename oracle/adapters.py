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

    def append_quantised(self, node, k, v, k_scales=None, v_scales=None, derive_scales=False):
        """bf16 tensors into an fp8 oracle tree (the library's quantising appends)."""
        ks = None if k_scales is None else raw_array(k_scales)
        vs = None if v_scales is None else raw_array(v_scales)
        self.tree.append_quantised(node, raw_array(k), raw_array(v), ks, vs, derive_scales=derive_scales)


class OracleDynamicSink:
    """The sink interface of the dynamic search driver (spex_workloads.dynamic) on top of an
    OracleTree: same seeded values, the oracle's own quantiser for decode tokens, attention only
    when `attend_every` says so (it is fp64 and slow), S_KV from its own token counts."""

    def __init__(self, shape, values, attend_every=0, sm_scale=None):
        self.shape, self.values = shape, values
        self.tree = OracleTree(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, shape.kv_dtype,
                               scale_block=shape.page_size)
        self.attend_every = attend_every
        self.sm_scale = sm_scale if sm_scale is not None else shape.head_dim ** -0.5
        self.results = {}                       # iteration -> (nodes, out, lse)
        self._last_tok = None

    def fork(self, parent, n):
        return self.tree.fork(parent, n)

    def prune(self, node):
        self.tree.prune(node)

    def path_kv_bytes(self, node):
        esz = {"bf16": 2, "fp8_e4m3": 1, "f32": 4}[self.shape.kv_dtype]
        tokens = pages = 0
        for u in self.tree.path(node):
            tokens += self.tree.n_tokens[u]
            pages += -(-self.tree.n_tokens[u] // self.shape.page_size)
        b = float(tokens) * 2.0 * self.shape.num_kv_heads * self.shape.head_dim * esz
        if self.shape.kv_dtype == "fp8_e4m3":
            b += float(pages) * 8.0 * self.shape.num_kv_heads
        return b

    def append_prompt(self, node, n, key):
        k, v = self.values.kv_run(key, 0, n)
        if self.shape.kv_dtype == "fp8_e4m3":
            # the oracle's own quantiser: page scales from the tokens, codes by its table search
            self.tree.append_quantised(node, raw_array(k.to(torch.bfloat16)), raw_array(v.to(torch.bfloat16)),
                                       derive_scales=True)
        else:
            self.tree.append(node, raw_array(k.to(torch.bfloat16)), raw_array(v.to(torch.bfloat16)))

    def append_tokens(self, nodes, keys, tok):
        k, v = self.values.kv_tokens(keys, tok)
        P = self.shape.page_size
        for i, u in enumerate(nodes):
            if self.shape.kv_dtype == "fp8_e4m3":
                s = None
                if self.tree.n_tokens[u] % P == 0:
                    s = np.full((1, self.shape.num_kv_heads), self.shape.fp8_scale, dtype=np.float32)
                self.tree.append_quantised(u, raw_array(k[i:i + 1]), raw_array(v[i:i + 1]), s, s)
            else:
                self.tree.append(u, raw_array(k[i:i + 1]), raw_array(v[i:i + 1]))
        self._last_tok = (list(keys), list(tok))

    def attend(self, nodes, iteration):
        if not self.attend_every or iteration % self.attend_every:
            return
        keys, tok = self._last_tok
        q = queries_fp64(self.values.queries(keys, tok))
        out, lse = self.tree.attention(list(nodes), None, q, self.sm_scale)
        self.results[iteration] = (list(nodes), out, lse)
