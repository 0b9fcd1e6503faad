"""CPU oracle for tree decode attention -- TEST INFRASTRUCTURE, not a product path.

Only tests, the smoke check and the benchmark's cpu_baseline leg may use this
module; the HIP library never does, and this module never touches the library.

What is computed.  The paper (Sec. 3.2, Sec. 4.1 insight 2, Sec. 4.3) states
that sibling Tree-of-Thought branches reuse the KV cache of their common
root-to-node prefix and that decoding is bound by KV-cache traffic; it gives no
formula for attention itself.  A prefix-sharing scheme must reproduce exactly
what each branch would compute alone, so the oracle is the plain definition:
for every requested node, lay the K/V of its root-to-node path out contiguously
and evaluate scaled-dot-product attention with grouped-query heads in fp64.

    T      = tokens on the path,  q_len queries attached to the node
    query i sees path positions 0 .. T - q_len + i          (causal among the q_len)
    or, with draft masks (token-level speculative decoding verifies a TREE of draft tokens,
    Sec. 6.5: token trees of 16 / 8 / 4 drafts): the q_len last tokens of the path are the
    drafts, query i sees every earlier position and draft j iff bit j of its mask is set
    (its ancestors in the draft tree and itself)
    kv head of query head h:  g = h // (Hq // Hkv)
    s_t = sm_scale * <q, K[t, g]>,  p = softmax(s),  out = sum_t p_t V[t, g],  lse = log sum_t e^{s_t}

The tree kept here has no pages: a node is a parent id plus contiguous arrays.
Inputs are decoded to fp64 from the exact bits the GPU receives: bf16 and fp8
(OCP e4m3fn, no infinities, 0x7F / 0xFF = NaN) are decoded by the bit-level
definitions below; an fp8 value is code * scale with one scale per block of
`scale_block` consecutive tokens of a node and per KV head, separately for K and V.

A cache that is quantised while tokens are appended (append_quantised) encodes
bf16 tokens with encode_e4m3 and the scale of the block they fall in; a block's
scale is fixed by the append that starts it.

Pins (tests/test_oracle_pins.py): brute-force loops, fp64 library attention on a
materialised branch, closed forms, softmax weights summing to one, identical
token paths, and the log-sum-exp merge identity over arbitrary partitions; for the
encoder: every code survives decode -> encode, midpoints go to the even code and
their fp32 neighbours to the nearer value, saturation, torch's own fp32 -> e4m3fn
cast on random values, exact rational arithmetic on a sample.
"""

from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

NO_NODE = -1


# ----------------------------------------------------------------------------- decoding
def decode_bf16(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> fp64 (a bf16 is the top half of an fp32)."""
    b = np.ascontiguousarray(bits).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def e4m3_table() -> np.ndarray:
    """All 256 e4m3fn values in fp64: 1 sign, 4 exponent (bias 7), 3 mantissa bits."""
    tab = np.empty(256, dtype=np.float64)
    for c in range(256):
        sign = -1.0 if c & 0x80 else 1.0
        e = (c >> 3) & 0xF
        m = c & 0x7
        if e == 0xF and m == 0x7:
            tab[c] = np.nan
        elif e == 0:
            tab[c] = sign * (m / 8.0) * 2.0 ** (-6)
        else:
            tab[c] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return tab


_E4M3 = e4m3_table()


def decode_e4m3(codes: np.ndarray) -> np.ndarray:
    return _E4M3[np.ascontiguousarray(codes).astype(np.uint8)]


def encode_e4m3(y: np.ndarray) -> np.ndarray:
    """Values -> e4m3fn codes for a cache that is quantised when tokens are appended: the
    representable value nearest to y, of two equally near ones the one with the even code (round
    to nearest even), magnitudes above 448 saturate to +-448, NaN stays NaN (0x7F | sign).
    Written as a search over the 127 finite non-negative values of the decode table, not as bit
    arithmetic."""
    y = np.asarray(y, dtype=np.float64)
    grid = _E4M3[:0x7F]                                   # codes 0x00 .. 0x7E, ascending
    a = np.minimum(np.abs(y), grid[-1])
    a = np.where(np.isnan(a), 0.0, a)
    hi = np.clip(np.searchsorted(grid, a, side="left"), 0, len(grid) - 1)    # first value >= a
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = a - grid[lo], grid[hi] - a
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = np.where(take_hi, hi, lo).astype(np.uint8)
    code = np.where(np.isnan(y), np.uint8(0x7F), code)
    return (code | np.where(np.signbit(y), np.uint8(0x80), np.uint8(0))).astype(np.uint8)


# ----------------------------------------------------------------------------- the tree
class OracleTree:
    """Forest of token steps.  Node ids are dense and follow creation order."""

    def __init__(self, num_q_heads: int, num_kv_heads: int, head_dim: int,
                 kv_dtype: str = "f32", scale_block: int = 16):
        assert num_q_heads % num_kv_heads == 0
        self.Hq, self.Hkv, self.D = num_q_heads, num_kv_heads, head_dim
        self.kv_dtype = kv_dtype
        self.scale_block = scale_block
        self.parent: List[int] = []
        self.children: List[List[int]] = []
        self.alive: List[bool] = []
        self.K: List[List[Optional[np.ndarray]]] = []   # per node: list of fp64 pieces [n, Hkv, D]
        self.V: List[List[Optional[np.ndarray]]] = []
        self.n_tokens: List[int] = []
        self._scales = {}                                # node -> (k_scales list, v_scales list)

    # -- mutation --------------------------------------------------------------------
    def fork(self, parent: int, n: int) -> List[int]:
        if parent != NO_NODE:
            self._check(parent)
        ids = []
        for _ in range(n):
            u = len(self.parent)
            self.parent.append(parent)
            self.children.append([])
            self.alive.append(True)
            self.K.append([])
            self.V.append([])
            self.n_tokens.append(0)
            if parent != NO_NODE:
                self.children[parent].append(u)
            ids.append(u)
        return ids

    def append(self, node: int, k, v, k_scales=None, v_scales=None, n_tokens=None) -> None:
        """k, v: [n, Hkv, D] as float arrays, uint16 bf16 bits or uint8 e4m3 codes
        (per kv_dtype); None = tokens whose values are unknown (count only)."""
        self._check(node)
        if any(self.alive[c] for c in self.children[node]):
            raise ValueError("append to a node that has children")
        if k is None:
            self.K[node].append(None)
            self.V[node].append(None)
            self.n_tokens[node] += int(n_tokens)
            return
        k = np.asarray(k)
        v = np.asarray(v)
        n = k.shape[0]
        assert k.shape == (n, self.Hkv, self.D) and v.shape == k.shape
        if self.kv_dtype == "f32":
            kd, vd = k.astype(np.float64), v.astype(np.float64)
        elif self.kv_dtype == "bf16":
            kd, vd = decode_bf16(k), decode_bf16(v)
        elif self.kv_dtype == "fp8_e4m3":
            kd = self._dequant(node, decode_e4m3(k), k_scales, 0)
            vd = self._dequant(node, decode_e4m3(v), v_scales, 1)
        else:
            raise ValueError(self.kv_dtype)
        self.K[node].append(kd)
        self.V[node].append(vd)
        self.n_tokens[node] += n

    def append_quantised(self, node: int, k_bits, v_bits, k_scales=None, v_scales=None,
                         derive_scales: bool = False) -> None:
        """fp8 cache filled from bf16 tokens (uint16 bit patterns [n, Hkv, D]): token j is encoded
        with the scale of the block of scale_block tokens it falls in.  A block this append starts
        takes the next row of k_scales / v_scales ([blocks this append starts, Hkv]) or, with
        derive_scales, max(amax / 448, 2^-40) where amax is the largest magnitude among the tokens
        this append puts into the block (per kv head, K and V separately, division in fp32); a
        block that already holds tokens keeps its scale and is never requantised.
        code = encode_e4m3(x * (1 / scale)) with the reciprocal and the product rounded to fp32,
        the precision in which the cache is written."""
        assert self.kv_dtype == "fp8_e4m3"
        self._check(node)
        B, start = self.scale_block, self.n_tokens[node]
        codes, made = [], []
        for which, bits, new in ((0, k_bits, k_scales), (1, v_bits, v_scales)):
            x = decode_bf16(np.asarray(bits)).astype(np.float32)
            blk = (start + np.arange(x.shape[0])) // B
            have = [r.astype(np.float32) for r in self._scales.get(node, ([], []))[which]]
            if derive_scales:
                assert new is None
                rows = []
                for b in range(len(have), int(blk.max()) + 1):          # the blocks this append starts
                    amax = np.abs(x[blk == b]).max(axis=(0, 2)).astype(np.float32)      # [Hkv]
                    rows.append(np.maximum(amax / np.float32(448.0), np.float32(2.0 ** -40)).astype(np.float32))
                new = np.stack(rows) if rows else None
            if new is not None:
                have += list(np.asarray(new, dtype=np.float32).reshape(-1, self.Hkv))
            assert blk.max() < len(have), "a started block needs a scale"
            sc = np.stack(have)[blk][:, :, None]                       # [n, Hkv, 1] fp32
            inv = (np.float32(1.0) / sc).astype(np.float32)
            codes.append(encode_e4m3((x * inv).astype(np.float32)))
            made.append(new)
        self.append(node, codes[0], codes[1], made[0], made[1])
        self.last_codes = codes                                        # for byte-level comparison
        self.last_scales = made

    def _dequant(self, node, x, new_scales, which):
        """Multiply codes by the scale of the block (of scale_block tokens of this node)
        each token falls in; new_scales holds the scales of the blocks this append starts."""
        B = self.scale_block
        store = self._scales.setdefault(node, ([], []))[which]
        if new_scales is not None:
            for row in np.asarray(new_scales, dtype=np.float32).reshape(-1, self.Hkv):
                store.append(row.astype(np.float64))
        start = self.n_tokens[node]
        blk = (start + np.arange(x.shape[0])) // B
        return x * np.stack(store)[blk][:, :, None]

    def prune(self, node: int) -> None:
        self._check(node)
        stack = [node]
        while stack:
            u = stack.pop()
            if self.alive[u]:
                self.alive[u] = False
                self.K[u], self.V[u] = [], []
                stack.extend(self.children[u])

    def _check(self, node: int) -> None:
        if not (0 <= node < len(self.parent)) or not self.alive[node]:
            raise KeyError(f"unknown or pruned node {node}")

    # -- reading ---------------------------------------------------------------------
    def path(self, node: int) -> List[int]:
        self._check(node)
        p = []
        while node != NO_NODE:
            p.append(node)
            node = self.parent[node]
        return p[::-1]

    def path_tokens(self, node: int) -> int:
        return sum(self.n_tokens[u] for u in self.path(node))

    def materialise(self, node: int):
        """Contiguous fp64 K, V of the root-to-node path: [T, Hkv, D] each."""
        ks, vs = [], []
        for u in self.path(node):
            for a, b in zip(self.K[u], self.V[u]):
                if a is None:
                    raise ValueError(f"node {u} holds tokens without values")
                ks.append(a)
                vs.append(b)
        if not ks:
            z = np.zeros((0, self.Hkv, self.D))
            return z, z.copy()
        return np.concatenate(ks, 0), np.concatenate(vs, 0)

    # -- attention -------------------------------------------------------------------
    def attention(self, leaves: Sequence[int], q_lens: Optional[Sequence[int]], q: np.ndarray,
                  sm_scale: float, return_weights: bool = False,
                  draft_masks: Optional[Sequence[int]] = None):
        """q: [sum(q_lens), Hq, D] fp64 (already decoded).  Returns out [.., Hq, D], lse [.., Hq]
        (and, on request, the list of per-query weight matrices [Hq, T_i]).
        draft_masks: one integer per query (request-major), bit j = the query sees draft token
        j of its request (path position T - q_len + j); None = the causal chain."""
        if q_lens is None:
            q_lens = [1] * len(leaves)
        q = np.asarray(q, dtype=np.float64)
        nq = int(sum(q_lens))
        assert q.shape == (nq, self.Hq, self.D)
        out = np.zeros((nq, self.Hq, self.D))
        lse = np.zeros((nq, self.Hq))
        weights = []
        G = self.Hq // self.Hkv
        row = 0
        for leaf, ql in zip(leaves, q_lens):
            K, V = self.materialise(leaf)
            T = K.shape[0]
            if ql < 1 or ql > T:
                raise ValueError("every query needs at least one visible token")
            for i in range(ql):
                if draft_masks is None:
                    vis = np.arange(T - ql + 1 + i)
                else:
                    mask = int(draft_masks[row])
                    if mask >> ql:
                        raise ValueError("mask bit beyond the request's drafts")
                    vis = np.array(list(range(T - ql)) + [T - ql + j for j in range(ql) if mask >> j & 1],
                                   dtype=np.int64)
                    if vis.size == 0:
                        raise ValueError("every query needs at least one visible token")
                Ti = vis.size
                w_all = np.zeros((self.Hq, Ti))
                for g in range(self.Hkv):
                    qg = q[row, g * G:(g + 1) * G, :]                 # [G, D]
                    s = sm_scale * (qg @ K[vis, g, :].T)              # [G, Ti]
                    m = s.max(axis=1, keepdims=True)
                    w = np.exp(s - m)
                    Z = w.sum(axis=1, keepdims=True)
                    p = w / Z
                    out[row, g * G:(g + 1) * G, :] = p @ V[vis, g, :]
                    lse[row, g * G:(g + 1) * G] = (m + np.log(Z))[:, 0]
                    w_all[g * G:(g + 1) * G] = p
                if return_weights:
                    weights.append(w_all)
                row += 1
        if return_weights:
            return out, lse, weights
        return out, lse


# ------------------------------------------------------------- partial attention and merge
def partial_attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, sm_scale: float):
    """Attention state of one query vector q [D] over a piece K, V [n, D]:
    (m, l, o) with m = max score, l = sum exp(s - m), o = sum exp(s - m) V (unnormalised).
    An empty piece gives (-inf, 0, 0)."""
    if K.shape[0] == 0:
        return -np.inf, 0.0, np.zeros(V.shape[1])
    s = sm_scale * (K @ q)
    m = s.max()
    w = np.exp(s - m)
    return m, w.sum(), w @ V


def lse_merge(parts):
    """Combine (m, l, o) states of disjoint pieces: with m = max m_j,
    l = sum l_j e^{m_j - m}, out = sum o_j e^{m_j - m} / l, lse = m + log l."""
    m = max(p[0] for p in parts)
    l = 0.0
    o = 0.0
    for mj, lj, oj in parts:
        if lj == 0.0:
            continue
        f = np.exp(mj - m)
        l = l + lj * f
        o = o + oj * f
    return o / l, m + np.log(l)
