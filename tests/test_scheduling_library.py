"""The C-ABI scheduling primitives (include/spex_sched.h) against the oracle: every integer
result bit for bit on seeded random inputs, scores to the last bit, error paths."""

import math

import numpy as np
import pytest

import paper_2605_10195_amd as spex
from paper_2605_10195_amd import binding as B
from oracle import scheduling as sch
from test_scheduling_oracle import random_search_tree


def test_rebase_widths_match_oracle():
    rng = np.random.default_rng(11)
    for trial in range(500):
        n = int(rng.integers(0, 40))
        R = rng.uniform(-2, 2, n).tolist() if trial % 3 else rng.integers(0, 4, n).astype(float).tolist()
        budget, T = int(rng.integers(0, 200)), float(rng.choice([0.05, 0.2, 1.0, 7.5]))
        assert B.spex_sched_rebase_widths(R, budget, T) == sch.rebase_widths(R, budget, T), (R, budget, T)
    # exact halves: four equal rewards and budget 2, 6, 10 -> 0.5, 1.5, 2.5 each
    for budget, want in ((2, 0), (6, 2), (10, 2), (14, 4)):
        assert B.spex_sched_rebase_widths([0.25] * 4, budget, 0.3) == [want] * 4


def to_lib(t):
    return B.SearchTree(t.parent, t.visits, t.value_sum, t.state, t.spec_reward, t.c)


def test_ucb_descent_and_speculative_selection_match_oracle():
    rng = np.random.default_rng(12)
    for trial in range(300):
        t = random_search_tree(rng, int(rng.integers(1, 60)), c=[0.0, 0.5, 1.4, None][trial % 4])
        lt = to_lib(t)
        assert B.spex_sched_ucb_select(lt) == sch.ucb_select(t)
        for k in (0, 1, 3, 8):
            assert B.spex_sched_dfs_speculate(lt, k) == sch.dfs_speculate(t, k), (trial, k)
    # a chain of single children; a root alone
    chain = sch.SearchTree([-1, 0, 1, 2], [3, 2, 1, 0], [1.0, 0.5, 0.2, 0.0])
    assert B.spex_sched_ucb_select(to_lib(chain)) == 3 and B.spex_sched_dfs_speculate(to_lib(chain), 2) == [3]
    lone = sch.SearchTree([-1], [0], [0.0])
    assert B.spex_sched_dfs_speculate(to_lib(lone), 3) == sch.dfs_speculate(lone, 3) == [0]


def test_budget_allocation_matches_oracle():
    rng = np.random.default_rng(13)
    for trial in range(500):
        n = int(rng.integers(0, 24))
        C = rng.integers(0, 17, n).tolist()
        P = rng.uniform(0, 1, n).tolist()
        S = (rng.uniform(0, 3e9, n) if trial % 2 else rng.integers(0, 5, n).astype(float)).tolist()
        Sw = 1.6e10 if trial % 2 else 2.0
        tau = float(rng.choice([0.0, 1e-11, 3e-11, -1e-11])) if trial % 2 else float(rng.uniform(-0.2, 0.5))
        kt = int(rng.integers(0, 256))
        k, scores = B.spex_sched_allocate_budget(C, P, S, Sw, tau, kt)
        k_ref, scores_ref = sch.allocate_budget(C, P, S, Sw, tau, kt)
        assert k == k_ref and scores == scores_ref, trial
    # 49 equal queries and 49 slots: 49 * (1 / 49) rounds below 1 in binary64, so nobody gets a slot --
    # the formula as it stands, in both implementations
    k, _ = B.spex_sched_allocate_budget([4] * 49, [0.5] * 49, [1.0] * 49, 1.0, 0.3, 49)
    assert k == sch.allocate_budget([4] * 49, [0.5] * 49, [1.0] * 49, 1.0, 0.3, 49)[0] == [0] * 49


def test_early_termination_matches_oracle():
    rng = np.random.default_rng(14)
    for trial in range(800):
        n = int(rng.integers(0, 30))
        ids = rng.integers(-3, 6, n).tolist()
        w = (rng.integers(0, 5, n) / 4.0 if trial % 2 else rng.uniform(0, 1, n)).tolist()   # quarters: exact ties
        t, alpha = int(rng.integers(0, 12)), float(rng.choice([0.0, 0.5, 1.0, 3.0]))
        assert B.spex_sched_early_termination(ids, w, t, alpha) == sch.early_termination(ids, w, t, alpha), trial


def test_path_kv_bytes_reads_the_page_table():
    for kv, esz in (("bf16", 2), ("fp8_e4m3", 1)):
        t = spex.SpexTree(8, 2, 64, 16, "bf16", kv, num_pages=16, host_only=True)
        (r,) = t.fork(-1, 1)
        t.append_step(r, None, None, n_tokens=40)               # 3 pages
        a, b = t.fork(r, 2)
        t.append_step(a, None, None, n_tokens=5)                # 1 page
        scales = 8 * 2 if kv == "fp8_e4m3" else 0
        assert B.spex_tree_path_kv_bytes(t, r) == 40 * 2 * 2 * 64 * esz + 3 * scales
        assert B.spex_tree_path_kv_bytes(t, a) == 45 * 2 * 2 * 64 * esz + 4 * scales
        assert B.spex_tree_path_kv_bytes(t, b) == B.spex_tree_path_kv_bytes(t, r)
        t.prune(b)
        with pytest.raises(spex.SpexError) as e:
            B.spex_tree_path_kv_bytes(t, b)
        assert e.value.name == "BAD_NODE"


def test_scheduling_error_paths():
    def bad(fn, *a):
        with pytest.raises(spex.SpexError) as e:
            fn(*a)
        assert e.value.name == "INVALID_ARG"
    bad(B.spex_sched_rebase_widths, [0.1, 0.2], 4, 0.0)
    bad(B.spex_sched_rebase_widths, [0.1, float("nan")], 4, 1.0)
    bad(B.spex_sched_rebase_widths, [0.1], -1, 1.0)
    bad(B.spex_sched_allocate_budget, [1], [1.5], [0.0], 1.0, 1.0, 4)          # hit rate above 1
    bad(B.spex_sched_allocate_budget, [-1], [0.5], [0.0], 1.0, 1.0, 4)
    bad(B.spex_sched_allocate_budget, [1], [0.5], [0.0], 1.0, float("inf"), 4)
    bad(B.spex_sched_early_termination, [1], [-0.5], 1, 0.5)
    bad(B.spex_sched_ucb_select, B.SearchTree([-1, 1], [1, 1], [0.0, 0.0]))       # parent[1] must be < 1
    bad(B.spex_sched_ucb_select, B.SearchTree([0], [1], [0.0]))                   # the root's parent is -1
    bad(B.spex_sched_ucb_select, B.SearchTree([-1, 0], [1, -1], [0.0, 0.0]))
    bad(B.spex_sched_ucb_select, B.SearchTree([-1, 0], [1, 1], [0.0, 0.0], state=[0, 7]))
    bad(B.spex_sched_dfs_speculate, B.SearchTree([-1], [1], [0.0], c=-1.0), 1)
