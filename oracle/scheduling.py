"""CPU oracle for the host-side scheduling primitives -- TEST INFRASTRUCTURE, not a product path.

Only tests (and the dynamic benchmark's cross-check leg) may use this module; the
library never does, and this module never touches the library.

The formulas are the paper's, written out with Python floats (IEEE binary64) and
plain loops, sums in index order, `math.exp` / `math.log` / `math.sqrt`:

  * rebase_widths      Sec. 2.1.1:  W_j = Round(B_i * softmax(R / T_b)_j)
  * ucb_select         Sec. 2.1.2:  a* = argmax_a Q(s, a) + c * sqrt(ln N(s) / N(s, a))
  * dfs_speculate      Sec. 4.2, Alg. 1: simulate the next k selections, skipping nodes under
                       expansion and folding in the rewards of finished speculations
  * allocate_budget    Sec. 4.3, Eq. 1-2: score_q = C_q * P_q * (S_w + S_KV(q)),
                       k_q = min(C_q, floor(k_total * softmax(tau * score)_q))
  * early_termination  Sec. 4.4, Eq. 3-4: n >= t and conf_1st - conf_2nd > alpha * avg(w_2nd)

Where the paper is silent the readings are: Round = nearest, halves to even; softmax
evaluated after subtracting the maximum; an unvisited child has infinite UCB; ties go to
the lowest index / smallest id; ln N(s) = 0 for N(s) = 0; Q = value_sum / visits (0 when
unvisited); in Alg. 1 "skip" counts a visit without reward along the node's root path
(otherwise the next simulated descent would return the same node), a finished speculation
backs its stored reward up along that path every time a descent ends at it, a selected node
counts a visit along its path and is treated as under expansion for the rest of the call;
at most k + 4 * n_nodes descents.

Pins (tests/test_oracle_pins.py): hand-computed values, uniform and winner-takes-all
limits, shift invariance, prefix consistency of the speculative list, and re-derivation
of every speculative choice by a single descent on an explicitly updated tree.
"""

from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

PLAIN, ACTIVE, SPEC_DONE = 0, 1, 2


def rebase_widths(rewards: Sequence[float], budget: int, temperature: float) -> List[int]:
    if not rewards:
        return []
    top = max(rewards)
    e = [math.exp((r - top) / temperature) for r in rewards]
    s = 0.0
    for x in e:
        s += x
    return [int(round(budget * (x / s))) for x in e]          # Python rounds halves to even


class SearchTree:
    """parent[u] < u, node 0 is the root; visits, value_sum, state, spec_reward per node."""

    def __init__(self, parent, visits, value_sum, state=None, spec_reward=None, c: float = 1.0):
        n = len(parent)
        self.parent = list(parent)
        self.visits = [int(v) for v in visits]
        self.value_sum = [float(v) for v in value_sum]
        self.state = list(state) if state is not None else [PLAIN] * n
        self.spec_reward = [float(v) for v in spec_reward] if spec_reward is not None else [0.0] * n
        self.c = float(c)
        self.children: List[List[int]] = [[] for _ in range(n)]
        for u in range(1, n):
            self.children[self.parent[u]].append(u)


def _descend(tree: SearchTree, visits: List[int], value_sum: List[float]) -> int:
    s = 0
    while True:
        kids = tree.children[s]
        if not kids:
            return s
        best, best_score = -1, 0.0
        log_n = math.log(visits[s]) if visits[s] > 0 else 0.0
        for a in kids:
            if visits[a] == 0:
                score = math.inf
            else:
                score = value_sum[a] / visits[a] + tree.c * math.sqrt(log_n / visits[a])
            if best < 0 or score > best_score:
                best, best_score = a, score
        s = best


def ucb_select(tree: SearchTree) -> int:
    return _descend(tree, tree.visits, tree.value_sum)


def dfs_speculate(tree: SearchTree, k: int) -> List[int]:
    n = len(tree.parent)
    visits, value_sum = list(tree.visits), list(tree.value_sum)
    selected: List[int] = []
    descents = 0

    def back_up(u: int, reward: Optional[float]) -> None:
        while u >= 0:
            visits[u] += 1
            if reward is not None:
                value_sum[u] += reward
            u = tree.parent[u]

    while len(selected) < k and descents < k + 4 * n:
        descents += 1
        node = _descend(tree, visits, value_sum)
        if tree.state[node] == SPEC_DONE:
            back_up(node, tree.spec_reward[node])
        elif tree.state[node] == ACTIVE or node in selected:
            back_up(node, None)
        else:
            selected.append(node)
            back_up(node, None)
    return selected


def allocate_budget(capacity: Sequence[int], hit_rate: Sequence[float], kv_bytes: Sequence[float],
                    param_bytes: float, tau: float, k_total: int) -> Tuple[List[int], List[float]]:
    n = len(capacity)
    scores = [capacity[q] * hit_rate[q] * (param_bytes + kv_bytes[q]) for q in range(n)]
    if n == 0:
        return [], []
    z = [tau * sc for sc in scores]
    top = max(z)
    e = [math.exp(x - top) for x in z]
    s = 0.0
    for x in e:
        s += x
    k = [min(int(capacity[q]), int(math.floor(k_total * (e[q] / s)))) for q in range(n)]
    return k, scores


def early_termination(answer_id: Sequence[int], weight: Sequence[float], t: int,
                      alpha: float) -> Tuple[bool, int]:
    conf, count = {}, {}
    for a, w in zip(answer_id, weight):
        conf[a] = conf.get(a, 0.0) + w
        count[a] = count.get(a, 0) + 1
    if not conf:
        return False, 0
    ranked = sorted(conf, key=lambda a: (-conf[a], a))
    first = ranked[0]
    conf2, avg2 = 0.0, 0.0
    if len(ranked) > 1:
        conf2 = conf[ranked[1]]
        avg2 = conf2 / count[ranked[1]]
    return (len(answer_id) >= t and conf[first] - conf2 > alpha * avg2), first
