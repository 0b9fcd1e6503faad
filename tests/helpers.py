"""Test-side helpers: an independent (torch) materialisation of branch K/V from a trace."""

import numpy as np
import torch

NO_NODE = -1


class RecordingSink:
    """Replay target that just records what every node was given; decodes with torch."""

    def __init__(self, wl):
        self.wl = wl
        self.parent, self.alive, self.kids = [], [], []
        self.k, self.v = [], []          # per node: list of fp64 tensors [n, Hkv, D]
        self.count = []
        self.k_scales, self.v_scales = {}, {}

    def fork(self, parent, n):
        ids = []
        for _ in range(n):
            u = len(self.parent)
            self.parent.append(parent)
            self.alive.append(True)
            self.kids.append([])
            self.k.append([])
            self.v.append([])
            self.count.append(0)
            if parent != NO_NODE:
                self.kids[parent].append(u)
            ids.append(u)
        return ids

    def prune(self, node):
        stack = [node]
        while stack:
            u = stack.pop()
            self.alive[u] = False
            stack.extend(self.kids[u])

    def _decode(self, node, x, new_scales, store):
        if x.dtype == torch.uint8:
            vals = x.cpu().view(torch.float8_e4m3fn).to(torch.float64)
            sc = store.setdefault(node, [])
            if new_scales is not None:
                sc.extend(new_scales.cpu().to(torch.float64).unbind(0))
            P = self.wl.page_size
            out = torch.empty_like(vals)
            for t in range(vals.shape[0]):
                out[t] = vals[t] * sc[(self.count[node] + t) // P][:, None]
            return out
        return x.cpu().to(torch.float64)

    def append(self, node, k, v, k_scales=None, v_scales=None, n_tokens=None):
        assert k is not None
        self.k[node].append(self._decode(node, k, k_scales, self.k_scales))
        self.v[node].append(self._decode(node, v, v_scales, self.v_scales))
        self.count[node] += k.shape[0]

    def branch(self, node):
        """fp64 K, V [T, Hkv, D] of the root-to-node path."""
        chain = []
        while node != NO_NODE:
            chain.append(node)
            node = self.parent[node]
        ks = [t for u in reversed(chain) for t in self.k[u]]
        vs = [t for u in reversed(chain) for t in self.v[u]]
        return torch.cat(ks, 0), torch.cat(vs, 0)


def error_metrics(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    max_abs = float(np.max(np.abs(got - ref))) if got.size else 0.0
    rel_l2 = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))
    return max_abs, rel_l2
