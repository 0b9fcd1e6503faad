"""Replay a trace into a tree implementation, generating K/V on the fly.

`sink` is any object with
    fork(parent: int, n: int) -> list[int]
    append(node: int, k, v, k_scales, v_scales) -> None
    prune(node: int) -> None
The library binding and the oracle's tree both offer these methods.  K/V come as
torch tensors [n_tokens, Hkv, D] on `device`: float32, bfloat16, or uint8 e4m3
codes accompanied by the scales of the pages the append newly starts
([n_new_pages, Hkv] fp32 each for K and V; None otherwise).
"""

from __future__ import annotations

from typing import Dict, List, Optional

import torch

from .quant import quantise_pages
from .rng import normal_values
from .trees import Workload

TAG_K, TAG_V, TAG_Q = 1, 2, 3


def _cast(x: torch.Tensor, dtype: str) -> torch.Tensor:
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return x.to(torch.bfloat16)
    raise ValueError(dtype)


def _gen_batch(wl: Workload, ops, device, pos0=None):
    """K and V (fp32) for a list of append ops, generated in one vectorised call."""
    lens = torch.tensor([op.n for op in ops], dtype=torch.int64, device=device)
    keys = torch.tensor([op.key for op in ops], dtype=torch.int64, device=device)
    tok0 = torch.tensor([op.tok0 for op in ops], dtype=torch.int64, device=device)
    total = int(lens.sum())
    starts = torch.cumsum(lens, 0) - lens
    node_keys = torch.repeat_interleave(keys, lens)
    tok = torch.arange(total, dtype=torch.int64, device=device) \
        - torch.repeat_interleave(starts, lens) + torch.repeat_interleave(tok0, lens)
    k = normal_values(wl.seed, TAG_K, node_keys, tok, wl.num_kv_heads, wl.head_dim,
                      wl.value_scale, device)
    v = normal_values(wl.seed, TAG_V, node_keys, tok, wl.num_kv_heads, wl.head_dim,
                      wl.value_scale, device)
    pf = wl.profile
    if pf is not None:
        if pf.k_ramp != 0.0 or pf.k_bias != 0.0:
            first = torch.tensor([pos0[op.node] for op in ops], dtype=torch.int64, device=device)
            pos = torch.repeat_interleave(first, lens) + tok
            k[:, :, 0] += (pf.k_ramp * pos.to(torch.float32) + pf.k_bias)[:, None]
        if pf.spikes:
            st = starts.tolist()
            for op, s0 in zip(ops, st):
                for t, val in pf.spikes.get(op.node, ()):
                    if op.tok0 <= t < op.tok0 + op.n:
                        k[s0 + t - op.tok0, :, 0] += val
        if pf.v_mult != 1.0:
            v = v * pf.v_mult
    return k, v, starts.tolist()


def replay(wl: Workload, sink, device="cpu", batch_tokens: Optional[int] = None,
           only_nodes=None) -> None:
    """Apply every op of `wl` to `sink`.

    only_nodes: optional set of node ids; appends to other nodes still happen (so
    that ids and page allocation stay the same) but carry k = v = None, which a
    sink may treat as "tokens whose values are never read".  The oracle uses this
    to hold values only for the paths it is asked about.
    """
    device = torch.device(device)
    if batch_tokens is None:
        per_tok = wl.num_kv_heads * wl.head_dim
        batch_tokens = max(1, ((1 << 28) if device.type == "cuda" else (1 << 23)) // per_tok)
    P = wl.page_size
    n_tokens: List[int] = []
    last_scale: Dict[int, tuple] = {}
    ready: Dict[int, tuple] = {}
    ops = wl.ops
    pos0 = wl.node_pos0() if wl.profile is not None else None
    for i, op in enumerate(ops):
        if op.kind == "fork":
            ids = sink.fork(op.node, op.n)
            assert list(ids) == list(range(len(n_tokens), len(n_tokens) + op.n)), \
                "sink does not hand out dense creation-order ids"
            n_tokens.extend([0] * op.n)
        elif op.kind == "prune":
            sink.prune(op.node)
        else:
            skip = only_nodes is not None and op.node not in only_nodes
            if skip:
                sink.append(op.node, None, None, None, None, n_tokens=op.n)
                n_tokens[op.node] += op.n
                continue
            if i not in ready:
                batch, tot, j = [], 0, i
                while j < len(ops) and (tot < batch_tokens or not batch):
                    o = ops[j]
                    if o.kind == "append" and (only_nodes is None or o.node in only_nodes):
                        batch.append(j)
                        tot += o.n
                    j += 1
                kb, vb, starts = _gen_batch(wl, [ops[j] for j in batch], device, pos0)
                for j, s in zip(batch, starts):
                    ready[j] = (kb[s:s + ops[j].n], vb[s:s + ops[j].n])
            k32, v32 = ready.pop(i)
            if wl.kv_dtype == "fp8_e4m3":
                slot = n_tokens[op.node] % P
                pk, pv = last_scale.get(op.node, (None, None))
                k, ks = quantise_pages(k32, slot, P, pk)
                v, vs = quantise_pages(v32, slot, P, pv)
                if ks.shape[0]:
                    last_scale[op.node] = (ks[-1].clone(), vs[-1].clone())
                sink.append(op.node, k, v, ks, vs)
            else:
                sink.append(op.node, _cast(k32, wl.kv_dtype).contiguous(),
                            _cast(v32, wl.kv_dtype).contiguous(), None, None)
            n_tokens[op.node] += op.n


def gen_queries(wl: Workload, device="cpu") -> torch.Tensor:
    """Query tensor [sum(q_lens), Hq, D] in the workload's q dtype, requested-node major."""
    device = torch.device(device)
    lens = torch.tensor(wl.q_lens, dtype=torch.int64, device=device)
    keys = torch.tensor(wl.q_keys, dtype=torch.int64, device=device)
    total = int(lens.sum())
    starts = torch.cumsum(lens, 0) - lens
    tok = torch.arange(total, dtype=torch.int64, device=device) - torch.repeat_interleave(starts, lens)
    q = normal_values(wl.seed, TAG_Q, torch.repeat_interleave(keys, lens), tok,
                      wl.num_q_heads, wl.head_dim, wl.value_scale, device)
    if wl.profile is not None and wl.profile.q0 is not None:
        q[:, :, 0] = wl.profile.q0
    return _cast(q, wl.q_dtype).contiguous()
