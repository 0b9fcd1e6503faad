"""The dynamic search driver (spex_workloads.dynamic): the C-ABI scheduling primitives and the
host page table drive exactly the trace the oracle's primitives and tree drive."""

import numpy as np
import pytest

import paper_2605_10195_amd as spex
from paper_2605_10195_amd import binding as B
from oracle import scheduling as sch
from oracle.adapters import OracleDynamicSink
from spex_workloads.dynamic import DynamicConfig, DynamicShape, DynamicValues, LibrarySink, RebaseSpexDriver


class LibSched:
    rebase_widths = staticmethod(B.spex_sched_rebase_widths)
    allocate_budget = staticmethod(B.spex_sched_allocate_budget)
    early_termination = staticmethod(B.spex_sched_early_termination)


class OracleSched:
    rebase_widths = staticmethod(sch.rebase_widths)
    allocate_budget = staticmethod(sch.allocate_budget)
    early_termination = staticmethod(sch.early_termination)


class Recorder:
    """Wraps a sink and writes down every tree operation."""

    def __init__(self, inner):
        self.inner, self.ops = inner, []

    def fork(self, parent, n):
        ids = self.inner.fork(parent, n)
        self.ops.append(("fork", parent, n, tuple(ids)))
        return ids

    def prune(self, node):
        self.ops.append(("prune", node))
        self.inner.prune(node)

    def append_prompt(self, node, n, key):
        self.ops.append(("prompt", node, n))
        self.inner.append_prompt(node, n, key)

    def append_tokens(self, nodes, keys, tok):
        self.ops.append(("tokens", tuple(nodes), tuple(tok)))
        self.inner.append_tokens(nodes, keys, tok)

    def attend(self, nodes, iteration):
        self.inner.attend(nodes, iteration)

    def path_kv_bytes(self, node):
        b = self.inner.path_kv_bytes(node)
        self.ops.append(("kv_bytes", node, b))
        return b


class CountingOracleSink(OracleDynamicSink):
    """Token counts only: no values are generated (the trace comparison needs none)."""

    def append_prompt(self, node, n, key):
        self.tree.append(node, None, None, n_tokens=n)

    def append_tokens(self, nodes, keys, tok):
        for u in nodes:
            self.tree.append(u, None, None, n_tokens=1)


@pytest.mark.parametrize("kv_dtype,seed", [("bf16", 11), ("fp8_e4m3", 12), ("bf16", 13)])
def test_library_and_oracle_drive_the_same_trace(kv_dtype, seed):
    cfg = DynamicConfig(n_queries=5, prompt=(40, 200), budget=8, max_depth=5, step=(4, 40), k_total=12, seed=seed)
    shape = DynamicShape(8, 2, 64, 16, kv_dtype)
    tree = spex.SpexTree(8, 2, 64, 16, "bf16", kv_dtype, num_pages=6000, host_only=True)
    lib_sink = Recorder(LibrarySink(tree, shape, None, B.spex_tree_path_kv_bytes, with_values=False))
    a = RebaseSpexDriver(cfg, lib_sink, LibSched)
    sa = a.run(2000)
    ora_sink = Recorder(CountingOracleSink(shape, None))
    b = RebaseSpexDriver(cfg, ora_sink, OracleSched)
    sb = b.run(2000)
    assert sa == sb and a.decisions == b.decisions and lib_sink.ops == ora_sink.ops
    # the run exercised everything: speculation with hits and misses, prunes, finished queries
    assert sa["finished_queries"] == cfg.n_queries and sa["spec_hits"] > 0 and sa["spec_misses"] > 0
    assert sa["prunes"] > 20 and any(d[0] == "budget" and sum(d[3]) > 0 for d in a.decisions)
    assert tree.stats()[0] == 0 and tree.stats()[1] == 0          # everything was returned to the pool


def test_dynamic_search_terminates_early_when_answers_agree():
    cfg = DynamicConfig(n_queries=6, prompt=(30, 60), budget=8, max_depth=8, step=(3, 20), p_terminal=0.6,
                        t_min=3, k_total=8, seed=21)
    shape = DynamicShape(8, 2, 64, 16, "bf16")
    sink = CountingOracleSink(shape, None)
    d = RebaseSpexDriver(cfg, sink, OracleSched)
    st = d.run(5000)
    assert st["finished_queries"] == 6 and st["early_terminations"] >= 1
    assert any(x[0] == "terminate" and x[3] for x in d.decisions)


# ------------------------------------------------------------------ depth-first search (Alg. 1)
class LibSchedDfs(LibSched):
    ucb_select = staticmethod(B.spex_sched_ucb_select)
    dfs_speculate = staticmethod(B.spex_sched_dfs_speculate)
    make_tree = staticmethod(B.SearchTree)


class OracleSchedDfs(OracleSched):
    ucb_select = staticmethod(sch.ucb_select)
    dfs_speculate = staticmethod(sch.dfs_speculate)
    make_tree = staticmethod(sch.SearchTree)


@pytest.mark.parametrize("kv_dtype,seed", [("bf16", 17), ("fp8_e4m3", 18)])
def test_mcts_library_and_oracle_drive_the_same_trace(kv_dtype, seed):
    from spex_workloads.dynamic import MctsConfig, MctsSpexDriver
    cfg = MctsConfig(n_queries=4, prompt=(40, 120), branch=3, rollouts=8, step=(3, 25), k_total=8,
                     k_per_query=3, seed=seed)
    shape = DynamicShape(8, 2, 64, 16, kv_dtype)
    tree = spex.SpexTree(8, 2, 64, 16, "bf16", kv_dtype, num_pages=6000, host_only=True)
    lib_sink = Recorder(LibrarySink(tree, shape, None, B.spex_tree_path_kv_bytes, with_values=False))
    a = MctsSpexDriver(cfg, lib_sink, LibSchedDfs)
    sa = a.run(3000)
    ora_sink = Recorder(CountingOracleSink(shape, None))
    b = MctsSpexDriver(cfg, ora_sink, OracleSchedDfs)
    sb = b.run(3000)
    assert sa == sb and a.decisions == b.decisions and lib_sink.ops == ora_sink.ops
    assert sa["finished_queries"] == cfg.n_queries and sa["spec_expansions"] > 0
    assert sa["spec_hits"] + sa["spec_waits"] > 0                 # predictions were used
    assert sa["max_depth"] >= 3 and tree.stats()[:2] == (0, 0)
