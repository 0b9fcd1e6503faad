"""Pins of the scheduling oracle (oracle/scheduling.py) against values worked out by hand from
the paper's formulas (Sec. 2.1.1, 2.1.2, Alg. 1, Eq. 1-4), limits and invariants."""

import math

import numpy as np
import pytest

from oracle import scheduling as sch


# ------------------------------------------------------------------ REBASE widths (Sec. 2.1.1)
def test_rebase_widths_hand_values_and_limits():
    T = 0.7
    # exp(R/T) in ratio 1 : 2 : 6 -> weights 1/9, 2/9, 6/9
    R = [0.3, 0.3 + T * math.log(2), 0.3 + T * math.log(6)]
    assert sch.rebase_widths(R, 9, T) == [1, 2, 6]
    assert sch.rebase_widths(R, 18, T) == [2, 4, 12]
    assert sch.rebase_widths([0.5] * 4, 16, 0.2) == [4, 4, 4, 4]
    assert sch.rebase_widths([0.5] * 4, 2, 0.2) == [0, 0, 0, 0]            # 0.5 each: halves go to even
    assert sch.rebase_widths([0.5] * 4, 6, 0.2) == [2, 2, 2, 2]            # 1.5 each
    assert sch.rebase_widths([0.1, 0.9], 8, 1e-3) == [0, 8]                # T_b -> 0: the best node takes all
    assert sch.rebase_widths([0.1, 0.9, 0.4], 9, 1e6) == [3, 3, 3]         # T_b -> inf: uniform
    assert sch.rebase_widths([], 5, 1.0) == [] and sch.rebase_widths([2.0], 7, 0.3) == [7]
    assert sch.rebase_widths([1000.0, 999.0], 10, 0.5) == sch.rebase_widths([1.0, 0.0], 10, 0.5)   # no overflow


def test_rebase_widths_shift_invariance_monotonicity_and_sum():
    rng = np.random.default_rng(1)
    for _ in range(200):
        n = int(rng.integers(1, 12))
        R = rng.uniform(0, 1, n).tolist()
        B, T = int(rng.integers(0, 40)), float(rng.uniform(0.05, 2))
        W = sch.rebase_widths(R, B, T)
        assert all(w >= 0 for w in W) and abs(sum(W) - B) <= n / 2 + 1e-9   # each term moves by at most 1/2
        order = np.argsort(R)
        assert all(W[order[i]] <= W[order[i + 1]] for i in range(n - 1))
        exact = [B * math.exp(r / T) / sum(math.exp(x / T) for x in R) for r in R]
        assert all(abs(w - e) <= 0.5 + 1e-9 for w, e in zip(W, exact))


# ------------------------------------------------------------------ UCB (Sec. 2.1.2)
def test_ucb_descent_hand_values():
    # root (N = 11) with children 1 (Q = .5, N = 10) and 2 (Q = .4, N = 1); c = 1:
    #   .5 + sqrt(ln 11 / 10) = 0.9897,  .4 + sqrt(ln 11 / 1) = 1.9485  -> child 2
    t = sch.SearchTree([-1, 0, 0], [11, 10, 1], [0.0, 5.0, 0.4], c=1.0)
    assert sch.ucb_select(t) == 2
    assert sch.ucb_select(sch.SearchTree([-1, 0, 0], [11, 10, 1], [0.0, 5.0, 0.4], c=0.0)) == 1   # greedy
    # break-even c: .5 + c * .48968 = .4 + c * 1.54851 -> c = 0.09444
    assert sch.ucb_select(sch.SearchTree([-1, 0, 0], [11, 10, 1], [0.0, 5.0, 0.4], c=0.0943)) == 1
    assert sch.ucb_select(sch.SearchTree([-1, 0, 0], [11, 10, 1], [0.0, 5.0, 0.4], c=0.0946)) == 2
    # an unvisited child is taken first, the lowest index among several
    assert sch.ucb_select(sch.SearchTree([-1, 0, 0, 0], [5, 5, 0, 0], [0.0, 5.0, 0.0, 0.0])) == 2
    # two levels: 0 -> {1, 2}, 1 -> {3, 4}; the descent ends at a childless node
    t = sch.SearchTree([-1, 0, 0, 1, 1], [20, 15, 5, 10, 5], [0.0, 12.0, 1.0, 9.0, 3.0], c=0.1)
    assert sch.ucb_select(t) == 3
    assert sch.ucb_select(sch.SearchTree([-1], [0], [0.0])) == 0


# ------------------------------------------------------------------ Alg. 1
def random_search_tree(rng, n, c=None):
    parent = [-1] + [int(rng.integers(0, u)) for u in range(1, n)]
    # visit counts consistent with a tree search: a node's count is at least its children's sum
    visits = [0] * n
    for u in range(n - 1, -1, -1):
        visits[u] += int(rng.integers(0, 4))
        if parent[u] >= 0:
            visits[parent[u]] += visits[u]
    value = [float(rng.uniform(0, 1)) * v for v in visits]
    state = [int(x) for x in rng.choice([0, 0, 0, 1, 2], size=n)]
    reward = [float(x) for x in rng.uniform(0, 1, n)]
    return sch.SearchTree(parent, visits, value, state, reward, c=float(rng.uniform(0, 2)) if c is None else c)


def test_dfs_speculate_first_choice_is_the_plain_descent_and_lists_are_prefix_consistent():
    rng = np.random.default_rng(2)
    for trial in range(60):
        t = random_search_tree(rng, int(rng.integers(1, 40)))
        plain = sch.SearchTree(t.parent, t.visits, t.value_sum, None, None, t.c)
        assert sch.dfs_speculate(plain, 1) == [sch.ucb_select(plain)]
        full = sch.dfs_speculate(t, 6)
        for k in range(6):
            assert sch.dfs_speculate(t, k) == full[:k]
        assert len(set(full)) == len(full)
        for u in full:
            assert t.children[u] == [] and t.state[u] == sch.PLAIN


def test_dfs_speculate_every_choice_rederived_by_single_descents():
    """Replay Alg. 1 with nothing but ucb_select on explicitly rebuilt trees."""
    rng = np.random.default_rng(3)
    for trial in range(40):
        t = random_search_tree(rng, int(rng.integers(2, 30)))
        want = sch.dfs_speculate(t, 5)
        visits, value, got, taken = list(t.visits), list(t.value_sum), [], set()
        for _ in range(5 + 4 * len(t.parent)):
            if len(got) == 5:
                break
            node = sch.ucb_select(sch.SearchTree(t.parent, visits, value, None, None, t.c))
            add = t.spec_reward[node] if t.state[node] == sch.SPEC_DONE else 0.0
            if t.state[node] == sch.PLAIN and node not in taken:
                got.append(node)
                taken.add(node)
            u = node
            while u >= 0:
                visits[u] += 1
                value[u] += add
                u = t.parent[u]
        assert got == want


def test_dfs_speculate_hand_case_skips_active_and_folds_finished_speculations():
    # root 0 (N = 6) -> 1 (N = 3, W = 2.4), 2 (N = 3, W = 1.2); c = 0: pure exploitation.
    # Q(1) = .8, Q(2) = .4.
    base = dict(parent=[-1, 0, 0], visits=[6, 3, 3], value_sum=[0.0, 2.4, 1.2])
    # plain tree: 1 is selected; a visit without reward makes Q(1) = 2.4 / 4 = .6 > .4: 1 again -> skipped
    # (already selected), Q(1) = 2.4 / 5 = .48: skipped again, 2.4 / 6 = .4: tie -> lowest index, skipped,
    # 2.4 / 7 < .4 -> 2.
    assert sch.dfs_speculate(sch.SearchTree(**base, c=0.0), 2) == [1, 2]
    # 1 under expansion: skipped four times, then 2; then 2's Q = 1.2 / 4 = .3 < 2.4 / 7: 1 is skipped
    # again ... only 2 can ever be returned
    act = sch.SearchTree(**base, state=[0, 1, 0], c=0.0)
    assert sch.dfs_speculate(act, 1) == [2] and sch.dfs_speculate(act, 2) == [2]
    # 1 is a finished speculation with reward 0: every fold lowers Q(1): 2.4/4, 2.4/5, 2.4/6 (tie -> 1), 2.4/7 -> 2
    done = sch.SearchTree(**base, state=[0, 2, 0], spec_reward=[0.0, 0.0, 0.0], c=0.0)
    assert sch.dfs_speculate(done, 1) == [2]
    # ... with reward 1 its Q only grows (3.4/4, 4.4/5, ..): nothing else is ever reached
    good = sch.SearchTree(**base, state=[0, 2, 0], spec_reward=[0.0, 1.0, 0.0], c=0.0)
    assert sch.dfs_speculate(good, 1) == []


# ------------------------------------------------------------------ Eq. 1-2
def test_budget_allocation_hand_values_and_limits():
    # scores: 2 * .5 * (1 + 1) = 2 and 4 * .5 * (1 + 3) = 8; tau = ln 2 / 6 -> weights 1/3, 2/3
    k, scores = sch.allocate_budget([2, 4], [0.5, 0.5], [1.0, 3.0], 1.0, math.log(2) / 6, 9)
    assert scores == [2.0, 8.0] and k == [2, 4]                            # floor(3) capped by C = 2; floor(6) by 4
    k, _ = sch.allocate_budget([20, 40], [0.05, 0.05], [1.0, 3.0], 1.0, math.log(2) / 6, 10)    # same scores
    assert k == [3, 6]                                                     # floor(3.33), floor(6.67): one slot unused
    assert sch.allocate_budget([5, 5, 5], [0.3, 0.3, 0.3], [7.0] * 3, 2.0, 0.4, 12)[0] == [4, 4, 4]
    assert sch.allocate_budget([5, 5, 5], [0.1, 0.9, 0.5], [1.0, 2.0, 3.0], 2.0, 0.0, 12)[0] == [4, 4, 4]   # tau = 0
    assert sch.allocate_budget([9, 9], [0.2, 0.8], [0.0, 0.0], 1.0, 1e3, 8)[0] == [0, 8]                   # sharp
    assert sch.allocate_budget([9, 9], [0.2, 0.8], [0.0, 0.0], 1.0, -1e3, 8)[0] == [8, 0]
    assert sch.allocate_budget([], [], [], 1.0, 1.0, 8) == ([], [])
    # model-sized numbers: 16 GB of parameters, KV of 0.1 - 2 GB, no overflow
    k, _ = sch.allocate_budget([8, 8, 8], [0.7, 0.6, 0.9], [1e8, 2e9, 5e8], 1.6e10, 1e-11, 16)
    assert sum(k) <= 16 and k[2] == max(k)


def test_budget_allocation_properties():
    rng = np.random.default_rng(4)
    for _ in range(200):
        n = int(rng.integers(1, 10))
        C = rng.integers(0, 12, n).tolist()
        P = rng.uniform(0, 1, n).tolist()
        S = rng.uniform(0, 5, n).tolist()
        kt, tau = int(rng.integers(0, 64)), float(rng.uniform(0, 0.3))
        k, scores = sch.allocate_budget(C, P, S, 1.5, tau, kt)
        assert all(0 <= k[q] <= C[q] for q in range(n)) and sum(k) <= kt
        for a in range(n):                      # a higher score never gets a smaller uncapped share
            for b in range(n):
                if scores[a] > scores[b] and k[a] < C[a]:
                    assert k[a] >= min(k[b], C[a])


# ------------------------------------------------------------------ Eq. 3-4
def test_early_termination_hand_values():
    ids, w = [7, 3, 7], [1.0, 0.5, 0.75]        # conf(7) = 1.75, conf(3) = .5, avg(w_2nd) = .5 (all exact)
    assert sch.early_termination(ids, w, 3, 0.5) == (True, 7)               # 1.25 > .25
    assert sch.early_termination(ids, w, 4, 0.5) == (False, 7)              # too few answers
    assert sch.early_termination(ids, w, 3, 2.5) == (False, 7)              # 1.25 > 1.25 fails (strict)
    assert sch.early_termination(ids, w, 3, 2.49) == (True, 7)
    assert sch.early_termination([1, 2], [0.5, 0.45], 1, 0.5) == (False, 1)  # .05 > .225 fails
    # 2nd hypothesis with many light answers: avg weight is what counts, not their number
    assert sch.early_termination([1, 2, 2, 2, 2], [1.0, 0.2, 0.2, 0.2, 0.2], 5, 0.5) == (True, 1)   # .2 > .1
    assert sch.early_termination([1, 2, 2, 2, 2], [0.85, 0.2, 0.2, 0.2, 0.2], 5, 0.5) == (False, 1)  # .05 > .1 fails
    assert sch.early_termination([4, 4], [0.3, 0.2], 2, 0.5) == (True, 4)    # one hypothesis: .5 > 0
    assert sch.early_termination([4, 4], [0.0, 0.0], 2, 0.5) == (False, 4)   # 0 > 0 fails
    assert sch.early_termination([], [], 0, 0.5) == (False, 0)
    assert sch.early_termination([5, 2], [0.4, 0.4], 1, 0.5) == (False, 2)   # tie: the smaller id is 1st
    # three hypotheses: only the top two enter
    assert sch.early_termination([1, 2, 3, 1], [0.5, 0.3, 0.29, 0.5], 4, 0.5) == (True, 1)   # 1.0 - .3 > .15
