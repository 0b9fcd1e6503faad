"""Invariants that pin the reference page-table / plan model (oracle/page_table_ref.py).

The model is what the C++ library is compared with bit for bit, so it is itself checked
here against properties that do not depend on how it is written.
"""

import numpy as np
import pytest

import spex_workloads as sw
from oracle.page_table_ref import OutOfPages, PageTableRef


def build(wl, num_pages=None, free_order=None):
    pt = PageTableRef(num_pages or wl.peak_pages(), wl.page_size, free_order)
    for op in wl.ops:
        if op.kind == "fork":
            pt.fork(op.node, op.n)
        elif op.kind == "append":
            pt.append(op.node, op.n)
        else:
            pt.prune(op.node)
    return pt


def check_ownership(pt):
    owner = {}
    for u, pages in enumerate(pt.pages):
        if not pt.alive[u]:
            assert pages == []
        assert len(pages) == -(-pt.tokens[u] // pt.P) or not pt.alive[u]
        for p in pages:
            assert p not in owner
            owner[p] = u
    live, used, free = pt.stats()
    assert used == len(owner) and used + free == pt.num_pages
    assert set(pt.free_list()).isdisjoint(owner) and len(set(pt.free_list())) == free


@pytest.mark.parametrize("seed", range(8))
def test_allocator_invariants_after_every_op(seed):
    wl = sw.random_trace(100 + seed, n_ops=80, max_tokens=50)
    rng = np.random.default_rng(seed)
    order = rng.permutation(wl.peak_pages() + 3).tolist()
    pt = PageTableRef(len(order), 16, order)
    for op in wl.ops:
        if op.kind == "fork":
            pt.fork(op.node, op.n)
        elif op.kind == "append":
            before = pt.free_list()
            new = pt.append(op.node, op.n)
            assert new == before[:len(new)]                 # pops in stack order
        else:
            sub_pages = []
            stack = [op.node]
            while stack:
                w = stack.pop()
                if pt.alive[w]:
                    sub_pages += pt.pages[w]
                    stack.extend(reversed(pt.children[w]))
            before = pt.free_list()
            pt.prune(op.node)
            assert pt.free_list() == sub_pages[::-1] + before   # pushed in visit order
            with pytest.raises(KeyError):
                pt.prune(op.node)                           # a pruned id stays rejected
        check_ownership(pt)


def test_first_pages_follow_free_order_and_oom_changes_nothing():
    pt = PageTableRef(6, 16, [4, 2, 5, 0, 1, 3])
    (r,) = pt.fork(-1, 1)
    assert pt.append(r, 17) == [4, 2]
    (c,) = pt.fork(r, 1)
    assert pt.append(c, 1) == [5]                          # child starts on a fresh page
    assert pt.append(c, 15) == []                          # fills that page
    state = (list(pt.free), [list(p) for p in pt.pages], list(pt.tokens))
    with pytest.raises(OutOfPages):
        pt.append(c, 16 * 3 + 1)
    assert state == (pt.free, pt.pages, pt.tokens)
    assert pt.path_pages(c) == ([4, 2, 5], [16, 1, 16])
    pt.prune(r)
    assert pt.stats() == (0, 0, 6)
    assert pt.free_list() == [5, 2, 4, 0, 1, 3]


def plan_of(wl, pt, pc, sc):
    return pt.plan(wl.leaves, wl.q_lens, wl.num_q_heads, wl.num_kv_heads, pc, sc)


@pytest.mark.parametrize("seed,pc,sc", [(s, pc, sc) for s in range(6) for pc, sc in ((1, 1), (3, 2), (64, 64))])
def test_plan_properties(seed, pc, sc):
    wl = sw.random_trace(200 + seed, n_ops=70, max_tokens=60, max_q_len=4)
    pt = build(wl)
    pl = plan_of(wl, pt, pc, sc)
    G = wl.num_q_heads // wl.num_kv_heads
    NQ = sum(wl.q_lens)
    # CSR equals path_pages
    for i, u in enumerate(wl.leaves):
        a, b = pl["leaf_indptr"][i], pl["leaf_indptr"][i + 1]
        assert (pl["leaf_pages"][a:b], pl["leaf_valid"][a:b]) == pt.path_pages(u)
    # limits
    qt = 0
    for u, ql in zip(wl.leaves, wl.q_lens):
        T = sum(pt.tokens[w] for w in pt.path(u))
        for i in range(ql):
            assert pl["qt_limit"][qt] == T - ql + 1 + i
            qt += 1
    # each distinct page on a requested path appears in exactly one task, once
    distinct = set(pl["leaf_pages"])
    assert sorted(pl["pg_id"]) == sorted(distinct)
    # tasks: for each query token, the pages of the tasks that list it, in task order, are its path
    n_tasks = len(pl["task_pbase"])
    per_qt = [[] for _ in range(NQ)]
    slots = set()
    pb = 0
    for t in range(n_tasks):
        a, n = pl["task_pg_begin"][t], pl["task_pg_count"][t]
        qa, qn = pl["task_qt_begin"][t], pl["task_qt_count"][t]
        assert n >= 1 and qn >= 1
        assert n <= (pc if t < pl["n_prefix_tasks"] else sc)
        assert pl["task_pbase"][t] == pb
        pb += qn * G * wl.num_kv_heads
        if t < pl["n_prefix_tasks"]:
            assert qn >= 2 or len(set(pl["qt_list"][qa:qa + qn])) >= 1
        rows = pl["qt_list"][qa:qa + qn]
        assert len(set(rows)) == len(rows)
        end_pos = pl["pg_pos"][a + n - 1] + pl["pg_valid"][a + n - 1]
        masked = any(v != 16 for v in pl["pg_valid"][a:a + n]) or \
            min(pl["qt_limit"][r] for r in rows) < end_pos
        assert pl["task_flags"][t] & 1 == int(masked)
        for r in rows:
            per_qt[r].append(t)
    assert pb == pl["n_partial_rows"]
    qt = 0
    for li, (u, ql) in enumerate(zip(wl.leaves, wl.q_lens)):
        pages, valid = pt.path_pages(u)
        pos = np.concatenate([[0], np.cumsum(valid)])[:-1].tolist()
        for i in range(ql):
            got_p, got_v, got_pos = [], [], []
            for t in per_qt[qt]:
                a, n = pl["task_pg_begin"][t], pl["task_pg_count"][t]
                got_p += pl["pg_id"][a:a + n]
                got_v += pl["pg_valid"][a:a + n]
                got_pos += pl["pg_pos"][a:a + n]
            assert (got_p, got_v, got_pos) == (pages, valid, pos)
            # merge list = the same tasks, slot bases disjoint and inside the task's block
            a, b = pl["part_indptr"][qt], pl["part_indptr"][qt + 1]
            assert b - a == len(per_qt[qt])
            for e, t in zip(range(a, b), per_qt[qt]):
                qa, qn = pl["task_qt_begin"][t], pl["task_qt_count"][t]
                r = pl["qt_list"][qa:qa + qn].index(qt)
                assert pl["part_base"][e] == pl["task_pbase"][t] + r * G
                assert pl["part_hstride"][e] == qn * G
                for g in range(wl.num_kv_heads):
                    for hh in range(G):
                        s = pl["part_base"][e] + g * pl["part_hstride"][e] + hh
                        assert s not in slots and s < pl["n_partial_rows"]
                        slots.add(s)
            qt += 1
    assert len(slots) == pl["n_partial_rows"]
    # final flag: exactly the suffix tasks that are their suffix's only chunk; merge_qt = the rest
    finals = set()
    for t in range(n_tasks):
        qa, qn = pl["task_qt_begin"][t], pl["task_qt_count"][t]
        rows = tuple(pl["qt_list"][qa:qa + qn])
        if t < pl["n_prefix_tasks"]:
            assert pl["task_flags"][t] & 2 == 0
            continue
        same = [u for u in range(pl["n_prefix_tasks"], n_tasks)
                if tuple(pl["qt_list"][pl["task_qt_begin"][u]:pl["task_qt_begin"][u] + pl["task_qt_count"][u]]) == rows]
        assert bool(pl["task_flags"][t] & 2) == (len(same) == 1)
        if len(same) == 1:
            finals.update(rows)
            # a final task is the last entry of each of its rows' merge lists
            for r in rows:
                assert per_qt[r][-1] == t
    assert pl["merge_qt"] == [q for q in range(NQ) if q not in finals]
    # groups: ascending ids, live >= 2, and their rows are the requests underneath
    assert pl["group_node"] == sorted(pl["group_node"])
    for w in pl["group_node"]:
        under = sum(1 for u in wl.leaves if w in pt.path(u))
        assert under >= 2 and pt.tokens[w] > 0


def test_sharing_counts_for_config_shapes():
    wl = sw.spec_at_scale(n_queries=3, prompt=64, step=32, branches=8)
    pt = build(wl)
    pl = plan_of(wl, pt, 1 << 20, 1 << 20)
    assert len(pl["pg_id"]) == wl.unique_kv_tokens() // 16
    # every root is a group holding all 8 branches of its query
    roots = [u for u in range(len(pt.parent)) if pt.parent[u] == -1]
    for r in roots:
        t = pl["group_node"].index(r)
        assert pl["task_qt_count"][t] == 8
    # each branch has a private one-step suffix
    assert len(pl["task_pbase"]) - pl["n_prefix_tasks"] == 24
    wl5 = sw.tot_with_drafts(n_queries=2, prompt=48, step=16)
    pl5 = plan_of(wl5, build(wl5), 1 << 20, 1 << 20)
    # depth-3 leaves are private: suffix = leaf step + the 6 drafts (one full + one partial page)
    suffix = range(pl5["n_prefix_tasks"], len(pl5["task_pbase"]))
    assert all(pl5["task_pg_count"][t] == 2 and pl5["task_qt_count"][t] == 6 for t in suffix)
    assert all(pl5["task_flags"][t] == 3 for t in suffix)        # masked and final
    assert all(pl5["task_flags"][t] == 0 for t in range(pl5["n_prefix_tasks"]))


def test_duplicate_and_interior_requests():
    pt = PageTableRef(16, 16)
    (r,) = pt.fork(-1, 1)
    pt.append(r, 20)
    a, b = pt.fork(r, 2)
    pt.append(a, 5)
    pl = pt.plan([a, a, r, b], [1, 2, 1, 1], 4, 2, 64, 64)     # b is empty, a twice, r interior
    assert pl["group_node"] == [r, a]
    assert pl["task_qt_count"][:2] == [5, 3]
    assert pl["n_prefix_tasks"] == 2 and len(pl["task_pbase"]) == 2     # no private suffix at all
    assert pl["qt_limit"] == [25, 24, 25, 20, 20]
    with pytest.raises(ValueError):
        pt.plan([a], [26], 4, 2, 64, 64)
