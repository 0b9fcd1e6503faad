"""A search that grows while it is served: breadth-first Tree-of-Thought (the REBASE rule) with
speculative expansion of finished nodes, over many user queries at once.

The static generators in trees.py freeze one moment of a search.  This driver produces the
whole life of the trees instead -- forks, one-token appends for every generating branch per
iteration, prunes of losers and mis-speculated branches, queries that end early -- which is
what ages the page allocator and what the cached plan has to survive (Sec. 3.1: steps of tens to
hundreds of tokens generated one at a time; Sec. 4.2: finished short branches are expanded
speculatively while the level waits for its stragglers; mis-speculated branches are terminated
at the barrier; Sec. 4.3: the speculative budget is split over queries; Sec. 4.4: a query stops
once its answers are decided).

The driver decides nothing itself.  Every scheduling decision comes from the `sched` object it
is given (the C-ABI primitives, or the oracle's, which lets a test run both and compare the
traces), every tree operation goes to the `sink` it is given (the HIP library, the oracle's tree,
or a recorder).  Rewards, step lengths and answers are seeded draws keyed by node id -- there is
no model and no reward model here.

sched:  rebase_widths(rewards, budget, temperature) -> [int]
        allocate_budget(capacity, hit_rate, kv_bytes, param_bytes, tau, k_total) -> ([int], [float])
        early_termination(answer_id, weight, t, alpha) -> (bool, int)
sink:   fork(parent, n) -> [ids];  prune(node);  append_prompt(node, n_tokens, key)
        append_tokens(nodes, keys, token_index)      one token for each node
        attend(nodes, iteration)                      decode attention for the tokens just appended
        path_kv_bytes(node) -> float                  S_KV of Eq. 1
"""

from __future__ import annotations

import time
from dataclasses import dataclass, field
from typing import Dict, List

from .rng import hash_key

NO_NODE = -1
_TAG_REWARD, _TAG_LEN, _TAG_ANSWER, _TAG_TERMINAL, _TAG_PROMPT, _TAG_NODE = 0x7265, 0x6C65, 0x616E, 0x7465, 0x7072, 0x6E6F6465


def _uniform(seed: int, tag: int, a: int, b: int = 0) -> float:
    """Seeded draw in [0, 1) keyed by (seed, tag, a, b); 53 bits."""
    return (hash_key(seed, tag, a, b) & ((1 << 53) - 1)) / float(1 << 53)


@dataclass
class DynamicConfig:
    n_queries: int = 16
    prompt: tuple = (256, 1024)          # prompt length, uniform
    budget: int = 16                     # B_i of the REBASE rule, every depth
    temperature: float = 0.2             # T_b
    max_depth: int = 6
    step: tuple = (8, 96)                # step length: lo + (hi - lo) * u^3, a long tail
    p_terminal: float = 0.25             # a node of depth >= 2 ends in an answer with this probability
    n_hypotheses: int = 4
    t_min: int = 4                       # t of Eq. 4
    alpha: float = 0.5                   # alpha of Eq. 4 (the paper's setting)
    tau: float = 2e-9                    # sharpness of Eq. 2 (scores are in bytes)
    param_bytes: float = 1.6e10          # S_w: an 8 B-parameter model in bf16
    k_total: int = 64                    # global speculative budget
    seed: int = 11


@dataclass
class _Node:
    query: int
    depth: int
    parent: int
    remaining: int
    spec: bool
    reward: float = -1.0                 # known once the step is finished
    terminal: bool = False
    done: bool = False
    alive: bool = True
    tokens: int = 0
    children: List[int] = field(default_factory=list)


class RebaseSpexDriver:
    def __init__(self, cfg: DynamicConfig, sink, sched):
        self.cfg, self.sink, self.sched = cfg, sink, sched
        self.nodes: Dict[int, _Node] = {}
        self.roots: List[int] = []
        self.level: Dict[int, List[int]] = {}          # query -> nodes of the level being generated
        self.depth: Dict[int, int] = {}
        self.answers: Dict[int, List[tuple]] = {}
        self.spec_made: Dict[int, int] = {}
        self.spec_hit: Dict[int, int] = {}
        self.live_queries: List[int] = []
        self.iteration = 0
        self.stats = dict(iterations=0, tokens=0, forks=0, prunes=0, spec_children=0, spec_hits=0,
                          spec_misses=0, early_terminations=0, finished_queries=0, max_generating=0)
        self.decisions: List[tuple] = []               # every scheduling decision, for trace comparison
        self._keys: Dict[int, int] = {}

    # ---- seeded properties of a node -----------------------------------------------------
    def _key(self, u: int) -> int:
        k = self._keys.get(u)
        if k is None:
            k = self._keys[u] = hash_key(self.cfg.seed, _TAG_NODE, u)
        return k

    def _step_len(self, u: int) -> int:
        lo, hi = self.cfg.step
        return lo + int((hi - lo) * _uniform(self.cfg.seed, _TAG_LEN, u) ** 3)

    def _reward(self, u: int) -> float:
        nd = self.nodes[u]
        base = self.nodes[nd.parent].reward if nd.parent != NO_NODE and self.nodes[nd.parent].reward >= 0 else 0.5
        return 0.5 * base + 0.5 * _uniform(self.cfg.seed, _TAG_REWARD, u)

    def _is_terminal(self, u: int) -> bool:
        nd = self.nodes[u]
        return nd.depth >= 2 and _uniform(self.cfg.seed, _TAG_TERMINAL, u) < self.cfg.p_terminal

    def _answer(self, u: int) -> int:
        # good branches agree on hypothesis 0, the others scatter
        if self.nodes[u].reward > 0.55:
            return 0
        return 1 + int(_uniform(self.cfg.seed, _TAG_ANSWER, u) * (self.cfg.n_hypotheses - 1))

    # ---- tree operations -----------------------------------------------------------------
    def _fork(self, parent: int, n: int, spec: bool) -> List[int]:
        if n <= 0:
            return []
        ids = self.sink.fork(parent, n)
        q = self.nodes[parent].query
        for u in ids:
            self.nodes[u] = _Node(q, self.nodes[parent].depth + 1, parent, 0, spec)
            self.nodes[u].remaining = self._step_len(u)
            self.nodes[parent].children.append(u)
        self.stats["forks"] += n
        if spec:
            self.stats["spec_children"] += n
            self.spec_made[q] += n
        return ids

    def _prune(self, u: int) -> None:
        """Remove u's subtree, then every ancestor (below the root) left without live children."""
        self.sink.prune(u)
        self.stats["prunes"] += 1
        stack = [u]
        while stack:
            w = stack.pop()
            self.nodes[w].alive = False
            stack.extend(c for c in self.nodes[w].children if self.nodes[c].alive)
        p = self.nodes[u].parent
        while p != NO_NODE and self.nodes[p].parent != NO_NODE and \
                not any(self.nodes[c].alive for c in self.nodes[p].children):
            self.sink.prune(p)
            self.stats["prunes"] += 1
            self.nodes[p].alive = False
            p = self.nodes[p].parent

    def start(self) -> None:
        cfg = self.cfg
        self.roots = self.sink.fork(NO_NODE, cfg.n_queries)
        for q, r in enumerate(self.roots):
            n = cfg.prompt[0] + int((cfg.prompt[1] - cfg.prompt[0] + 1) * _uniform(cfg.seed, _TAG_PROMPT, q))
            self.nodes[r] = _Node(q, 0, NO_NODE, 0, False, reward=0.5, done=True, tokens=n)
            self.sink.append_prompt(r, n, self._key(r))
            self.answers[q], self.spec_made[q], self.spec_hit[q] = [], 0, 0
            self.depth[q] = 0
            self.level[q] = self._fork(r, cfg.budget, False)
            self.live_queries.append(q)

    # ---- one decode iteration of every generating branch ------------------------------------
    def step(self) -> bool:
        generating = sorted(u for u, nd in self.nodes.items() if nd.alive and nd.remaining > 0)
        if not generating and not self.live_queries:
            return False
        if generating:
            self.sink.append_tokens(generating, [self._key(u) for u in generating],
                                    [self.nodes[u].tokens for u in generating])
            self.sink.attend(generating, self.iteration)
            self.stats["tokens"] += len(generating)
            self.stats["max_generating"] = max(self.stats["max_generating"], len(generating))
            for u in generating:
                nd = self.nodes[u]
                nd.tokens += 1
                nd.remaining -= 1
                if nd.remaining == 0:
                    nd.done = True
                    nd.reward = self._reward(u)
                    nd.terminal = self._is_terminal(u)
        self.iteration += 1
        self.stats["iterations"] = self.iteration
        self._speculate()
        for q in list(self.live_queries):
            if all(self.nodes[u].done for u in self.level[q]):
                self._barrier(q)
        return True

    # ---- Sec. 4.2 (BFS) + Sec. 4.3: expand finished nodes while the level waits ---------------
    def _speculate(self) -> None:
        cfg = self.cfg
        waiting = [q for q in self.live_queries if any(not self.nodes[u].done for u in self.level[q])]
        cand = {q: [u for u in self.level[q] if self.nodes[u].done and not self.nodes[u].terminal]
                for q in waiting}
        waiting = [q for q in waiting if cand[q] and self.depth[q] + 1 < cfg.max_depth]
        if not waiting:
            return
        capacity = [len(cand[q]) for q in waiting]       # the speculative budget matches the finished nodes
        hit_rate = [(self.spec_hit[q] + 1) / (self.spec_made[q] + 2) for q in waiting]
        kv = [self.sink.path_kv_bytes(max(cand[q], key=lambda u: (self.nodes[u].reward, -u))) for q in waiting]
        k, _ = self.sched.allocate_budget(capacity, hit_rate, kv, cfg.param_bytes, cfg.tau, cfg.k_total)
        self.decisions.append(("budget", self.iteration, tuple(waiting), tuple(k)))
        for q, k_q in zip(waiting, k):
            if k_q <= 0:
                continue
            widths = self.sched.rebase_widths([self.nodes[u].reward for u in cand[q]], k_q, cfg.temperature)
            self.decisions.append(("spec_widths", self.iteration, q, tuple(widths)))
            for u, w in zip(cand[q], widths):
                have = sum(1 for c in self.nodes[u].children if self.nodes[c].alive)
                self._fork(u, w - have, True)

    # ---- the level is complete: the real expansion, verification of the speculation -----------
    def _barrier(self, q: int) -> None:
        cfg = self.cfg
        level = self.level[q]
        for u in level:
            if self.nodes[u].terminal:
                self.answers[q].append((self._answer(u), self.nodes[u].reward))
        open_nodes = [u for u in level if not self.nodes[u].terminal]
        stop, _ = self.sched.early_termination([a for a, _ in self.answers[q]], [w for _, w in self.answers[q]],
                                               cfg.t_min, cfg.alpha)
        self.decisions.append(("terminate", self.iteration, q, bool(stop)))
        self.depth[q] += 1
        if stop or not open_nodes or self.depth[q] >= cfg.max_depth:
            self.stats["early_terminations"] += int(bool(stop))
            self.stats["finished_queries"] += 1
            self._prune(self.roots[q])
            self.live_queries.remove(q)
            return
        widths = self.sched.rebase_widths([self.nodes[u].reward for u in open_nodes], cfg.budget, cfg.temperature)
        self.decisions.append(("widths", self.iteration, q, tuple(widths)))
        nxt: List[int] = []
        for u in level:
            if self.nodes[u].terminal:
                self._prune(u)                    # its answer is recorded; the branch is finished
        for u, w in zip(open_nodes, widths):
            spec = [c for c in self.nodes[u].children if self.nodes[c].alive]
            keep, drop = spec[:w], spec[w:]
            for c in drop:                        # mis-speculation: not selected by the real frontier
                self._prune(c)
            self.stats["spec_hits"] += len(keep)
            self.stats["spec_misses"] += len(drop)
            self.spec_hit[q] += len(keep)
            for c in keep:
                self.nodes[c].spec = False
            nxt += keep + self._fork(u, w - len(keep), False)
            if w == 0 and self.nodes[u].alive:    # (dropping its last child has already removed it)
                self._prune(u)
        if not nxt:
            self.stats["finished_queries"] += 1
            self._prune(self.roots[q])
            self.live_queries.remove(q)
            return
        self.level[q] = nxt

    def run(self, max_iterations: int) -> dict:
        if not self.roots:
            self.start()
        while self.iteration < max_iterations and self.step():
            pass
        return self.stats


# ---- values and sinks --------------------------------------------------------------------------
@dataclass
class DynamicShape:
    num_q_heads: int = 32
    num_kv_heads: int = 8
    head_dim: int = 128
    page_size: int = 16
    kv_dtype: str = "bf16"               # "bf16" | "fp8_e4m3"
    value_scale: float = 0.5
    fp8_scale: float = 2.0 ** -7         # scale given to every page a decode token starts (fp8)


class DynamicValues:
    """Seeded K / V / Q of the dynamic search: token t of node u is keyed by (node key, t), so
    every sink receives the same bits whatever order it is driven in."""

    def __init__(self, shape: DynamicShape, seed: int, device="cpu", table_rows: int = 0):
        """table_rows > 0 (a power of two): decode tokens and queries are rows (key + token) mod
        table_rows of tables drawn once -- one gather per tensor instead of a hash per element;
        for timing runs, where only the cost of making the values matters."""
        import torch
        from .replay import TAG_K, TAG_Q, TAG_V
        self.shape, self.seed, self.device = shape, seed, torch.device(device)
        self._tags = (TAG_K, TAG_V, TAG_Q)
        self._tables = None
        if table_rows:
            assert table_rows & (table_rows - 1) == 0
            rows = torch.arange(table_rows, dtype=torch.int64, device=self.device)
            zero = torch.zeros_like(rows)
            self._tables = {tag: self._draw(tag, rows, zero, heads).to(torch.bfloat16)
                            for tag, heads in ((TAG_K, shape.num_kv_heads), (TAG_V, shape.num_kv_heads),
                                               (TAG_Q, shape.num_q_heads))}
            self._mask = table_rows - 1

    def _draw(self, tag, keys, tok, heads):
        import torch
        from .rng import normal_values
        keys = torch.as_tensor(keys, dtype=torch.int64, device=self.device)
        tok = torch.as_tensor(tok, dtype=torch.int64, device=self.device)
        if self._tables is not None and tag in self._tables:
            return self._tables[tag][(keys + tok) & self._mask]
        return normal_values(self.seed, tag, keys, tok, heads, self.shape.head_dim, self.shape.value_scale,
                             self.device)

    def kv_run(self, key: int, first: int, n: int):
        """fp32 K, V [n, Hkv, D] of tokens first .. first + n - 1 of one node."""
        import torch
        tok = torch.arange(first, first + n, dtype=torch.int64, device=self.device)
        keys = torch.full((n,), key, dtype=torch.int64, device=self.device)
        return (self._draw(self._tags[0], keys, tok, self.shape.num_kv_heads),
                self._draw(self._tags[1], keys, tok, self.shape.num_kv_heads))

    def kv_tokens(self, keys, tok):
        """bf16 K, V [len(keys), Hkv, D]: one token for each node."""
        import torch
        return (self._draw(self._tags[0], keys, tok, self.shape.num_kv_heads).to(torch.bfloat16),
                self._draw(self._tags[1], keys, tok, self.shape.num_kv_heads).to(torch.bfloat16))

    def queries(self, keys, tok):
        import torch
        return self._draw(self._tags[2], keys, tok, self.shape.num_q_heads).to(torch.bfloat16).contiguous()


class LibrarySink:
    """Drives a tree object with the binding's methods (fork, prune, append_step, append_tokens,
    decode_attention); `path_bytes(tree, node)` is the page-table read of S_KV."""

    def __init__(self, tree, shape: DynamicShape, values: DynamicValues, path_bytes, sm_scale=None,
                 with_values: bool = True):
        self.tree, self.shape, self.values, self._path_bytes = tree, shape, values, path_bytes
        self.sm_scale = sm_scale if sm_scale is not None else shape.head_dim ** -0.5
        self.with_values = with_values
        self.last = None                          # (nodes, q, out, lse) of the latest attention call
        self.plan_states = {0: 0, 1: 0, 2: 0}
        # host seconds spent inside the tree object's calls, by kind (what the harness itself
        # costs -- drawing values, the search bookkeeping -- is the rest of the wall time)
        self.call_seconds = {"fork_prune": 0.0, "append": 0.0, "attention": 0.0}

    def _timed(self, kind, fn, *args, **kwargs):
        t0 = time.perf_counter()
        try:
            return fn(*args, **kwargs)
        finally:
            self.call_seconds[kind] += time.perf_counter() - t0

    def fork(self, parent, n):
        return self._timed("fork_prune", self.tree.fork, parent, n)

    def prune(self, node):
        self._timed("fork_prune", self.tree.prune, node)

    def path_kv_bytes(self, node):
        return self._path_bytes(self.tree, node)

    def append_prompt(self, node, n, key):
        if not self.with_values:
            self._timed("append", self.tree.append_step, node, None, None, n_tokens=n)
            return
        import torch
        k, v = self.values.kv_run(key, 0, n)
        if self.shape.kv_dtype == "fp8_e4m3":
            # bf16 tokens in; the library's scatter kernel derives the page scales and encodes
            self._timed("append", self.tree.append_step, node, k.to(torch.bfloat16).contiguous(),
                        v.to(torch.bfloat16).contiguous(), quantize=True)
        else:
            self._timed("append", self.tree.append_step, node, k.to(torch.bfloat16).contiguous(),
                        v.to(torch.bfloat16).contiguous())

    def append_tokens(self, nodes, keys, tok):
        if not self.with_values:
            self._timed("append", self.tree.append_tokens, nodes, None, None)
            return
        import torch
        k, v = self.values.kv_tokens(keys, tok)
        if self.shape.kv_dtype == "fp8_e4m3":
            s = torch.full((len(nodes), self.shape.num_kv_heads), self.shape.fp8_scale, dtype=torch.float32,
                           device=k.device)
            self._timed("append", self.tree.append_tokens, nodes, k.contiguous(), v.contiguous(), s, s,
                        quantize=True)
        else:
            self._timed("append", self.tree.append_tokens, nodes, k.contiguous(), v.contiguous())
        self._last_tok = (list(keys), list(tok))

    def attend(self, nodes, iteration):
        if not self.with_values:
            return
        keys, tok = self._last_tok
        q = self.values.queries(keys, tok)
        out, lse = self._timed("attention", self.tree.decode_attention, nodes, None, q, self.sm_scale)
        self.plan_states[self.tree.last_launch_info()["plan_rebuilt"]] += 1
        self.last = (list(nodes), q, out, lse)


# ---- depth-first search (MCTS) with speculative expansion: Sec. 4.2, Alg. 1 ---------------------
@dataclass
class MctsConfig:
    n_queries: int = 16
    prompt: tuple = (256, 1024)
    branch: int = 3                      # children created by one expansion
    rollouts: int = 10                   # primary expansions per query (the paper runs 5 / 10)
    c: float = 1.4                       # exploration constant of UCB
    step: tuple = (8, 96)
    p_terminal: float = 0.2              # a child of depth >= 3 ends in an answer
    n_hypotheses: int = 4
    t_min: int = 4
    alpha: float = 0.5
    tau: float = 2e-9
    param_bytes: float = 1.6e10
    k_total: int = 32                    # speculative expansions in flight, all queries together
    k_per_query: int = 4                 # C_q: how far ahead one query is simulated
    seed: int = 17


class MctsSpexDriver:
    """One search tree per query, kept as the parallel arrays spex_search_tree_t points to.  A
    primary expansion takes the node a UCB descent ends at and generates `branch` children below
    it; when they are finished their rewards are backed up.  Meanwhile the nodes the search is
    predicted to select next (sched.dfs_speculate) are expanded speculatively: such a node is
    ACTIVE while its children generate and SPEC_DONE afterwards, its children stay outside the
    arrays.  When a later descent ends at a SPEC_DONE node its children are adopted at once (a
    hit: no generation, no waiting); when it ends at an ACTIVE node the query waits for it.
    Nothing is pruned before the query ends: an unused prediction stays a candidate (Sec. 4.2).

    sched: ucb_select(tree) -> node, dfs_speculate(tree, k) -> [nodes], allocate_budget(...),
    early_termination(...), where `tree` is built by sched.make_tree(parent, visits, value_sum,
    state, spec_reward, c)."""

    PLAIN, ACTIVE, SPEC_DONE = 0, 1, 2

    def __init__(self, cfg: MctsConfig, sink, sched):
        self.cfg, self.sink, self.sched = cfg, sink, sched
        self.q: List[dict] = []
        self.gen: Dict[int, dict] = {}            # KV node -> {query, remaining, tokens}
        self.iteration = 0
        self.stats = dict(iterations=0, tokens=0, expansions=0, spec_expansions=0, spec_hits=0, spec_waits=0,
                          early_terminations=0, finished_queries=0, max_generating=0, max_depth=0)
        self.decisions: List[tuple] = []
        self._keys: Dict[int, int] = {}

    def _key(self, u):
        k = self._keys.get(u)
        if k is None:
            k = self._keys[u] = hash_key(self.cfg.seed, _TAG_NODE, u)
        return k

    def start(self):
        cfg = self.cfg
        roots = self.sink.fork(NO_NODE, cfg.n_queries)
        for i, r in enumerate(roots):
            n = cfg.prompt[0] + int((cfg.prompt[1] - cfg.prompt[0] + 1) * _uniform(cfg.seed, _TAG_PROMPT, i))
            self.sink.append_prompt(r, n, self._key(r))
            # search arrays; kv[s] = KV-tree node of search node s; pending[s] = children being generated
            self.q.append(dict(root=r, parent=[-1], visits=[0], value=[0.0], state=[0], spec_reward=[0.0], kv=[r],
                               depth=[0], pending={}, waiting=None, rollouts=0, answers=[], live=True,
                               spec_made=0, spec_hit=0))

    def _tree(self, st):
        return self.sched.make_tree(st["parent"], st["visits"], st["value"], st["state"], st["spec_reward"],
                                    self.cfg.c)

    def _expand(self, qi, s, speculative):
        """Fork `branch` children below search node s and start generating their steps."""
        st = self.q[qi]
        kids = self.sink.fork(st["kv"][s], self.cfg.branch)
        lo, hi = self.cfg.step
        for u in kids:
            n = lo + int((hi - lo) * _uniform(self.cfg.seed, _TAG_LEN, u) ** 3)
            self.gen[u] = dict(query=qi, remaining=n, tokens=0)
        st["pending"][s] = dict(kids=list(kids), left=len(kids), speculative=speculative)
        st["state"][s] = self.ACTIVE
        self.stats["expansions" if not speculative else "spec_expansions"] += 1
        if speculative:
            st["spec_made"] += 1

    def _adopt(self, qi, s):
        """The children of s enter the arrays with their rewards backed up along the path."""
        st = self.q[qi]
        info = st["pending"].pop(s)
        st["state"][s] = self.PLAIN
        for u in info["kids"]:
            d = st["depth"][s] + 1
            r = 0.5 * (st["value"][s] / st["visits"][s] if st["visits"][s] else 0.5) \
                + 0.5 * _uniform(self.cfg.seed, _TAG_REWARD, u)
            c = len(st["parent"])
            st["parent"].append(s)
            st["visits"].append(1)
            st["value"].append(r)
            st["state"].append(self.PLAIN)
            st["spec_reward"].append(0.0)
            st["kv"].append(u)
            st["depth"].append(d)
            self.stats["max_depth"] = max(self.stats["max_depth"], d)
            a = s
            while a >= 0:
                st["visits"][a] += 1
                st["value"][a] += r
                a = st["parent"][a]
            if d >= 3 and _uniform(self.cfg.seed, _TAG_TERMINAL, u) < self.cfg.p_terminal:
                hyp = 0 if r > 0.55 else 1 + int(_uniform(self.cfg.seed, _TAG_ANSWER, u) * (self.cfg.n_hypotheses - 1))
                st["answers"].append((hyp, r))

    def _finish(self, qi):
        st = self.q[qi]
        st["live"] = False
        for u in [u for u, g in self.gen.items() if g["query"] == qi]:
            del self.gen[u]
        self.sink.prune(st["root"])
        self.stats["finished_queries"] += 1

    def _advance(self, qi):
        """Primary search of query qi: select, adopt finished speculations, expand."""
        st, cfg = self.q[qi], self.cfg
        while st["live"] and st["waiting"] is None:
            stop, _ = self.sched.early_termination([a for a, _ in st["answers"]], [w for _, w in st["answers"]],
                                                   cfg.t_min, cfg.alpha)
            if stop or st["rollouts"] >= cfg.rollouts:
                self.decisions.append(("finish", self.iteration, qi, bool(stop)))
                self.stats["early_terminations"] += int(bool(stop))
                self._finish(qi)
                return
            s = self.sched.ucb_select(self._tree(st))
            self.decisions.append(("select", self.iteration, qi, s, st["state"][s]))
            st["rollouts"] += 1
            if st["state"][s] == self.SPEC_DONE:          # predicted and already generated: a hit
                self.stats["spec_hits"] += 1
                st["spec_hit"] += 1
                self._adopt(qi, s)
                continue
            if st["state"][s] == self.ACTIVE:             # being generated speculatively: wait for it
                self.stats["spec_waits"] += 1
                st["pending"][s]["speculative"] = False
                st["waiting"] = s
                return
            self._expand(qi, s, False)
            st["waiting"] = s

    def _speculate(self):
        cfg = self.cfg
        live = [i for i, st in enumerate(self.q) if st["live"]]
        in_flight = sum(1 for i in live for p in self.q[i]["pending"].values() if p["speculative"] and p["left"] > 0)
        room = cfg.k_total - in_flight
        if room <= 0 or not live:
            return
        capacity = [cfg.k_per_query] * len(live)
        hit = [(self.q[i]["spec_hit"] + 1) / (self.q[i]["spec_made"] + 2) for i in live]
        kv = [self.sink.path_kv_bytes(self.q[i]["kv"][self.q[i]["waiting"]] if self.q[i]["waiting"] is not None
                                      else self.q[i]["root"]) for i in live]
        k, _ = self.sched.allocate_budget(capacity, hit, kv, cfg.param_bytes, cfg.tau, room)
        self.decisions.append(("budget", self.iteration, tuple(live), tuple(k)))
        for qi, k_q in zip(live, k):
            if k_q <= 0:
                continue
            picks = self.sched.dfs_speculate(self._tree(self.q[qi]), k_q)
            self.decisions.append(("speculate", self.iteration, qi, tuple(picks)))
            for s in picks:
                self._expand(qi, s, True)

    def step(self) -> bool:
        if not any(st["live"] for st in self.q):
            return False
        generating = sorted(self.gen)
        if generating:
            self.sink.append_tokens(generating, [self._key(u) for u in generating],
                                    [self.gen[u]["tokens"] for u in generating])
            self.sink.attend(generating, self.iteration)
            self.stats["tokens"] += len(generating)
            self.stats["max_generating"] = max(self.stats["max_generating"], len(generating))
            for u in generating:
                g = self.gen[u]
                g["tokens"] += 1
                g["remaining"] -= 1
                if g["remaining"] == 0:
                    del self.gen[u]
                    st = self.q[g["query"]]
                    s = next(s for s, p in st["pending"].items() if u in p["kids"])
                    p = st["pending"][s]
                    p["left"] -= 1
                    if p["left"] == 0:
                        if p["speculative"]:
                            st["state"][s] = self.SPEC_DONE
                            st["spec_reward"][s] = sum(_uniform(self.cfg.seed, _TAG_REWARD, k) for k in p["kids"]) \
                                / len(p["kids"])
                        else:
                            self._adopt(g["query"], s)
                            if st["waiting"] == s:
                                st["waiting"] = None
        self.iteration += 1
        self.stats["iterations"] = self.iteration
        for qi, st in enumerate(self.q):
            if st["live"] and st["waiting"] is None:
                self._advance(qi)
        self._speculate()
        return True

    def run(self, max_iterations: int) -> dict:
        if not self.q:
            self.start()
            for qi in range(len(self.q)):
                self._advance(qi)
            self._speculate()
        while self.iteration < max_iterations and self.step():
            pass
        return self.stats
