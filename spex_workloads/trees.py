"""Fork / append / prune traces that build the synthetic search trees.

A trace is a list of TreeOp.  Node ids are dense integers handed out in creation
order (a fork of n children creates ids next .. next+n-1), which is the id rule
of the library and of the oracle's own tree, so one trace drives both.

The five named generators stand in for the tree shapes of the paper's
workloads (Sec. 6.1, Table 1: BFS methods of width 8/16, MCTS methods with 5/10
rollouts; Sec. 3.1: steps of tens to hundreds of tokens, skewed trees deeper
than 10; Sec. 6.5: token-level draft budgets of 4-16).  No dataset, model or
reward is involved: survivors, widths and lengths are drawn from a seeded
generator.
"""

from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from .rng import hash_key

NO_NODE = -1


@dataclass
class TreeOp:
    kind: str          # "fork" | "append" | "prune"
    node: int          # fork: parent (NO_NODE = new root); append / prune: the node
    n: int = 0         # fork: number of children; append: number of tokens
    key: int = 0       # append: random-stream key of the node's tokens
    tok0: int = 0      # append: index, within that stream, of the first appended token


@dataclass
class ValueProfile:
    """Structure laid over the i.i.d. values of a workload, so that tests can shape the scores
    (inputs only -- which scores result is for the library and the oracle to work out):
      q0      every query's dim 0 is set to this value (None: left as drawn);
      k_ramp  added to dim 0 of every K token: k_ramp * (the token's position on its root path);
      k_bias  added to dim 0 of every K token;
      spikes  node -> [(token index inside the node, value added to dim 0 of that K token)];
      v_mult  V is multiplied by this (a power of two keeps it exact).
    With q0 = b, the score of a token moves by sm_scale * b * (what was added to its K)."""
    q0: Optional[float] = None
    k_ramp: float = 0.0
    k_bias: float = 0.0
    spikes: Optional[dict] = None
    v_mult: float = 1.0


@dataclass
class Workload:
    name: str
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    q_dtype: str                 # "f32" | "bf16"
    kv_dtype: str                # "f32" | "bf16" | "fp8_e4m3"
    value_scale: float           # power of two applied to the N(0,1) draws
    seed: int
    ops: List[TreeOp] = field(default_factory=list)
    leaves: List[int] = field(default_factory=list)     # nodes queried in the measured launch
    q_lens: List[int] = field(default_factory=list)     # queries per requested node
    q_keys: List[int] = field(default_factory=list)     # random-stream key of each node's queries
    sm_scale: float = 0.0
    n_trees: int = 0
    # visibility mask of every query token among its request's q_len drafts (bit k = draft k is
    # seen), or None for the causal chain
    draft_masks: Optional[List[int]] = None
    profile: Optional[ValueProfile] = None

    def __post_init__(self):
        if self.sm_scale == 0.0:
            self.sm_scale = 1.0 / math.sqrt(self.head_dim)

    # ---- bookkeeping helpers (no attention arithmetic) -------------------------------
    def node_tokens(self):
        """Final token count, parent and liveness per node id after replaying the trace."""
        tokens, parent, alive = [], [], []
        children = []
        for op in self.ops:
            if op.kind == "fork":
                for _ in range(op.n):
                    tokens.append(0)
                    parent.append(op.node)
                    alive.append(True)
                    children.append([])
                    if op.node != NO_NODE:
                        children[op.node].append(len(tokens) - 1)
            elif op.kind == "append":
                tokens[op.node] += op.n
            elif op.kind == "prune":
                stack = [op.node]
                while stack:
                    u = stack.pop()
                    if alive[u]:
                        alive[u] = False
                        stack.extend(children[u])
        return tokens, parent, alive

    def node_pos0(self) -> List[int]:
        """Path position of every node's first token (tokens of its ancestors)."""
        tokens, parent, _ = self.node_tokens()
        pos0 = [0] * len(tokens)
        for u in range(len(tokens)):          # ids follow creation order: a parent precedes its children
            pos0[u] = 0 if parent[u] == NO_NODE else pos0[parent[u]] + tokens[parent[u]]
        return pos0

    def peak_pages(self) -> int:
        """Largest number of pages in use at any point of the trace."""
        P = self.page_size
        tokens, alive, children = [], [], []
        used = peak = 0
        for op in self.ops:
            if op.kind == "fork":
                for _ in range(op.n):
                    tokens.append(0)
                    alive.append(True)
                    children.append([])
                    if op.node != NO_NODE:
                        children[op.node].append(len(tokens) - 1)
            elif op.kind == "append":
                before = -(-tokens[op.node] // P)
                tokens[op.node] += op.n
                used += -(-tokens[op.node] // P) - before
                peak = max(peak, used)
            else:
                stack = [op.node]
                while stack:
                    u = stack.pop()
                    if alive[u]:
                        alive[u] = False
                        used -= -(-tokens[u] // P)
                        stack.extend(children[u])
        return peak

    def path_tokens(self, node: int) -> int:
        tokens, parent, _ = self.node_tokens()
        t = 0
        while node != NO_NODE:
            t += tokens[node]
            node = parent[node]
        return t

    def unique_kv_tokens(self) -> int:
        """Distinct tokens on the root-to-node paths of the requested nodes."""
        tokens, parent, _ = self.node_tokens()
        seen = set()
        for leaf in self.leaves:
            u = leaf
            while u != NO_NODE and u not in seen:
                seen.add(u)
                u = parent[u]
        return sum(tokens[u] for u in seen)

    def flat_kv_tokens(self) -> int:
        """Tokens read if every requested path were stored privately (no sharing)."""
        tokens, parent, _ = self.node_tokens()
        total = 0
        for leaf in self.leaves:
            u = leaf
            while u != NO_NODE:
                total += tokens[u]
                u = parent[u]
        return total

    def kv_bytes_per_token(self) -> float:
        esz = {"f32": 4, "bf16": 2, "fp8_e4m3": 1}[self.kv_dtype]
        b = 2.0 * self.num_kv_heads * self.head_dim * esz
        if self.kv_dtype == "fp8_e4m3":
            b += 2.0 * self.num_kv_heads * 4 / self.page_size   # K and V scale per (page, head)
        return b


class _Builder:
    """Hands out node ids exactly as the library and the oracle tree do."""

    def __init__(self, wl: Workload):
        self.wl = wl
        self.next_id = 0
        self.tokens: List[int] = []

    def fork(self, parent: int, n: int) -> List[int]:
        self.wl.ops.append(TreeOp("fork", parent, n))
        ids = list(range(self.next_id, self.next_id + n))
        self.next_id += n
        self.tokens.extend([0] * n)
        return ids

    def append(self, node: int, n: int, key: Optional[int] = None):
        if key is None:
            key = hash_key(self.wl.seed, 0x6E6F6465, node)
        self.wl.ops.append(TreeOp("append", node, n, key, self.tokens[node]))
        self.tokens[node] += n

    def prune(self, node: int):
        self.wl.ops.append(TreeOp("prune", node))

    def request(self, node: int, q_len: int = 1, key: Optional[int] = None):
        self.wl.leaves.append(node)
        self.wl.q_lens.append(q_len)
        self.wl.q_keys.append(hash_key(self.wl.seed, 0x71756572, node) if key is None else key)


def tiny_tree(seed: int = 1) -> Workload:
    """Config 1: one tree, a 256-token prompt, one fork into 4 branches of 64 tokens; fp32."""
    wl = Workload("tiny_tree", 8, 2, 64, 16, "f32", "f32", 1.0, seed, n_trees=1)
    b = _Builder(wl)
    (root,) = b.fork(NO_NODE, 1)
    b.append(root, 256)
    for c in b.fork(root, 4):
        b.append(c, 64)
        b.request(c)
    return wl


def bfs_tot(seed: int = 2, n_queries: int = 32, prompt: int = 512, step: int = 128,
            width: int = 16, keep: int = 4, depth: int = 5,
            heads=(32, 8, 128), kv_dtype: str = "bf16", q_dtype: str = "bf16") -> Workload:
    """Config 2: BFS frontier search.  Per query: a prompt node, `width` children, and at each
    of the depths 1..depth-1 a seeded uniform draw keeps `keep` of the `width` frontier nodes;
    each survivor forks width/keep children.  Losers are pruned, and so is any ancestor left
    without a live descendant.  Every step holds exactly `step` tokens."""
    wl = Workload("bfs_tot", heads[0], heads[1], heads[2], 16, q_dtype, kv_dtype, 0.5, seed,
                  n_trees=n_queries)
    b = _Builder(wl)
    rng = np.random.default_rng(seed)
    fan = width // keep
    for _ in range(n_queries):
        (root,) = b.fork(NO_NODE, 1)
        b.append(root, prompt)
        parent_of = {root: NO_NODE}
        kids = {root: []}
        frontier = b.fork(root, width)
        for c in frontier:
            parent_of[c] = root
            kids[c] = []
            kids[root].append(c)
            b.append(c, step)
        for _d in range(1, depth):
            chosen = sorted(rng.choice(len(frontier), size=keep, replace=False).tolist())
            survivors = [frontier[i] for i in chosen]
            live = set()
            for s in survivors:
                u = s
                while u != NO_NODE and u not in live:
                    live.add(u)
                    u = parent_of[u]
            pruned = set()
            for loser in frontier:
                if loser in live:
                    continue
                u = loser
                while parent_of[u] not in live:
                    u = parent_of[u]
                if u not in pruned:
                    pruned.add(u)
                    b.prune(u)
            frontier = []
            for s in survivors:
                cs = b.fork(s, fan)
                for c in cs:
                    parent_of[c] = s
                    kids[c] = []
                    kids[s].append(c)
                    b.append(c, step)
                frontier.extend(cs)
        for leaf in frontier:
            b.request(leaf)
    return wl


def mcts_skewed(seed: int = 3, n_queries: int = 64, prompt=(256, 1024), step=(32, 256),
                max_depth: int = 10, max_leaves: int = 64,
                heads=(28, 4, 128), kv_dtype: str = "bf16", q_dtype: str = "bf16") -> Workload:
    """Config 3: skewed trees grown by a seeded random walk.  Target leaf count per query is
    min(max_leaves, floor(2^U[0, log2 max_leaves])) (heavy tailed); 70 % of the expansions
    extend the current best path, the others hit a uniformly chosen node shallower than
    max_depth; an expansion forks 1..4 children with one step of U{step} tokens each."""
    wl = Workload("mcts_skewed", heads[0], heads[1], heads[2], 16, q_dtype, kv_dtype, 0.5, seed,
                  n_trees=n_queries)
    b = _Builder(wl)
    rng = np.random.default_rng(seed)
    for _ in range(n_queries):
        (root,) = b.fork(NO_NODE, 1)
        b.append(root, int(rng.integers(prompt[0], prompt[1] + 1)))
        target = min(max_leaves, int(2.0 ** rng.uniform(0.0, math.log2(max_leaves))))
        depth = {root: 0}
        nkids = {root: 0}
        nodes = [root]
        tip = root
        leaves = 1
        while leaves < target:
            open_nodes = [u for u in nodes if depth[u] < max_depth]
            if not open_nodes:
                break
            if depth[tip] < max_depth and rng.random() < 0.7:
                u = tip
            else:
                u = open_nodes[int(rng.integers(0, len(open_nodes)))]
            room = max_leaves - leaves + (1 if nkids[u] == 0 else 0)
            c = min(int(rng.integers(1, 5)), room)
            if c <= 0:
                break
            cs = b.fork(u, c)
            leaves += c - (1 if nkids[u] == 0 else 0)
            nkids[u] += c
            for ch in cs:
                depth[ch] = depth[u] + 1
                nkids[ch] = 0
                nodes.append(ch)
                b.append(ch, int(rng.integers(step[0], step[1] + 1)))
            if u == tip:
                tip = cs[0]
        for u in nodes:
            if nkids[u] == 0:
                b.request(u)
    return wl


def spec_at_scale(seed: int = 4, n_queries: int = 256, prompt: int = 2048, step: int = 256,
                  branches: int = 32, max_fork_depth: int = 4,
                  heads=(64, 8, 128), kv_dtype: str = "bf16", q_dtype: str = "bf16") -> Workload:
    """Config 4: per query a primary chain prompt -> P1 -> P2 -> P3 (one step each) and
    `branches` speculative branches; a branch draws d = min(Geometric(0.5), 4) and hangs, with
    one private step, below the primary node of depth d-1."""
    wl = Workload("spec_at_scale", heads[0], heads[1], heads[2], 16, q_dtype, kv_dtype, 0.5, seed,
                  n_trees=n_queries)
    b = _Builder(wl)
    rng = np.random.default_rng(seed)
    for _ in range(n_queries):
        (root,) = b.fork(NO_NODE, 1)
        b.append(root, prompt)
        chain = [root]
        for _d in range(1, max_fork_depth):
            (p,) = b.fork(chain[-1], 1)
            b.append(p, step)
            chain.append(p)
        ds = np.minimum(rng.geometric(0.5, size=branches), max_fork_depth)
        for d in ds.tolist():
            (br,) = b.fork(chain[d - 1], 1)
            b.append(br, step)
            b.request(br)
    return wl


def tot_with_drafts(seed: int = 5, n_queries: int = 64, prompt: int = 1024, step: int = 128,
                    depth: int = 3, drafts: int = 6,
                    heads=(40, 8, 128), kv_dtype: str = "fp8_e4m3", q_dtype: str = "bf16",
                    token_trees: bool = False) -> Workload:
    """Config 5: per query a binary tree prompt -> 2 -> 4 -> 8 with one step per node; every
    leaf then receives `drafts` draft tokens that are verified by `drafts` causal queries, or,
    with token_trees, by queries that see the drafts along a seeded token tree."""
    wl = Workload("tot_with_drafts", heads[0], heads[1], heads[2], 16, q_dtype, kv_dtype, 0.5, seed,
                  n_trees=n_queries)
    b = _Builder(wl)
    for _ in range(n_queries):
        (root,) = b.fork(NO_NODE, 1)
        b.append(root, prompt)
        level = [root]
        for _d in range(depth):
            nxt = []
            for u in level:
                cs = b.fork(u, 2)
                for c in cs:
                    b.append(c, step)
                nxt.extend(cs)
            level = nxt
        for leaf in level:
            b.append(leaf, drafts)
            b.request(leaf, drafts)
    return with_draft_trees(wl) if token_trees else wl


def step_prefill(seed: int = 6, n_queries: int = 32, prompt: int = 512, step: int = 128, width: int = 16,
                 keep: int = 4, depth: int = 5, heads=(32, 8, 128), kv_dtype: str = "bf16",
                 q_dtype: str = "bf16") -> Workload:
    """The tree of config 2 at the moment its newest steps are scored: a process reward model reads
    every frontier node's whole step (Sec. 2.1: rewards come from a reward model; Sec. 6.1 runs one
    next to the generator), i.e. q_len = step queries per leaf, causal among themselves, over the
    shared root-to-parent prefix."""
    wl = bfs_tot(seed, n_queries, prompt, step, width, keep, depth, heads, kv_dtype, q_dtype)
    wl.name = "step_prefill"
    wl.q_lens = [step] * len(wl.leaves)
    return wl


def draft_tree_masks(seed: int, key: int, n: int) -> List[int]:
    """A seeded draft token tree of n tokens (Sec. 6.5 verifies token trees of 4-16 drafts): draft
    0 is the root, the parent of draft j > 0 is drawn from the drafts before it; the mask of a
    draft has the bits of its ancestors and its own."""
    rng = np.random.default_rng([seed & 0xFFFFFFFF, key & 0xFFFFFFFF, (key >> 32) & 0xFFFFFFFF, n])
    masks = [1]
    for j in range(1, n):
        masks.append(masks[int(rng.integers(0, j))] | (1 << j))
    return masks


def with_draft_trees(wl: Workload) -> Workload:
    """The same workload with every request's q_len queries arranged as a seeded token tree."""
    assert all(ql <= 32 for ql in wl.q_lens)
    wl.draft_masks = []
    for key, ql in zip(wl.q_keys, wl.q_lens):
        wl.draft_masks += draft_tree_masks(wl.seed, key, ql)
    wl.name += "_token_trees"
    return wl


def random_trace(seed: int, heads=(8, 2, 64), kv_dtype: str = "bf16", q_dtype: str = "bf16",
                 n_ops: int = 60, max_tokens: int = 70, max_q_len: int = 1,
                 n_roots: int = 2, p_prune: float = 0.12, request_interior: bool = True,
                 value_scale: float = 0.5) -> Workload:
    """Small random tree with ragged step lengths, prunes, empty nodes, re-appends to the same
    node and (optionally) queries on interior nodes; used by the parity and page-table tests."""
    wl = Workload(f"random_{seed}", heads[0], heads[1], heads[2], 16, q_dtype, kv_dtype,
                  value_scale, seed)
    b = _Builder(wl)
    rng = np.random.default_rng(seed)
    parent, kids, alive = {}, {}, {}

    def new_nodes(par, n):
        ids = b.fork(par, n)
        for c in ids:
            parent[c] = par
            kids[c] = []
            alive[c] = True
            if par != NO_NODE:
                kids[par].append(c)
        return ids

    for r in new_nodes(NO_NODE, n_roots):
        b.append(r, int(rng.integers(1, max_tokens + 1)))
    for _ in range(n_ops):
        live = [u for u in alive if alive[u]]
        if not live:
            for r in new_nodes(NO_NODE, 1):
                b.append(r, int(rng.integers(1, max_tokens + 1)))
            continue
        x = rng.random()
        u = live[int(rng.integers(0, len(live)))]
        if x < p_prune and len(live) > 2:
            stack = [u]
            while stack:
                w = stack.pop()
                alive[w] = False
                stack.extend(k for k in kids[w] if alive[k])
            b.prune(u)
        elif x < 0.55:
            for c in new_nodes(u, int(rng.integers(1, 4))):
                if rng.random() < 0.85:            # some children stay empty
                    b.append(c, int(rng.integers(1, max_tokens + 1)))
        else:
            if not any(alive[k] for k in kids[u]):  # append only to childless nodes
                b.append(u, int(rng.integers(1, max_tokens + 1)))
    wl.n_trees = sum(1 for u in alive if parent[u] == NO_NODE and alive[u])
    tokens, par, _ = wl.node_tokens()

    def path_len(u):
        t = 0
        while u != NO_NODE:
            t += tokens[u]
            u = par[u]
        return t

    for u in sorted(alive):
        if not alive[u]:
            continue
        is_leaf = not any(alive[k] for k in kids[u])
        if not is_leaf and not (request_interior and rng.random() < 0.2):
            continue
        T = path_len(u)
        if T == 0:
            continue
        b.request(u, int(rng.integers(1, min(max_q_len, T) + 1)))
    return wl


WORKLOADS = {
    "tiny_tree": tiny_tree,
    "bfs_tot": bfs_tot,
    "mcts_skewed": mcts_skewed,
    "spec_at_scale": spec_at_scale,
    "tot_with_drafts": tot_with_drafts,
    "step_prefill": step_prefill,
}
