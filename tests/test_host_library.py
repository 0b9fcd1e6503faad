"""Host side of the library through the C ABI, on CPU: exported symbols, page table, allocator,
prune and the per-launch plan, all bit-exact against the reference model."""

import ctypes
import os
import re

import numpy as np
import pytest

import spex_workloads as sw
from oracle.page_table_ref import OutOfPages, PageTableRef
import paper_2605_10195_amd as spex
from paper_2605_10195_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(binding.LIB_PATH)
    for fname, exports in (("spex_tree.h", binding.EXPORTS), ("spex_sched.h", binding.SCHED_EXPORTS)):
        header = open(os.path.join(ROOT, "include", fname)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)             # declarations, not prose
        declared = set(re.findall(r"\b(spex_[a-z0-9_]+)\s*\(", header))
        assert declared == set(exports), fname
        for name in declared:
            assert hasattr(lib, name), name
    assert binding.lib.spex_status_string(4) == b"page pool exhausted"


def host_tree(wl, num_pages, free_order=None, **kw):
    return spex.SpexTree(wl.num_q_heads, wl.num_kv_heads, wl.head_dim, wl.page_size, wl.q_dtype,
                         wl.kv_dtype, num_pages=num_pages, free_order=free_order, host_only=True, **kw)


def replay_both(wl, tree, ref, check_every_op=False):
    for op in wl.ops:
        if op.kind == "fork":
            assert tree.fork(op.node, op.n) == ref.fork(op.node, op.n)
        elif op.kind == "append":
            assert tree.append_new_pages(op.node, op.n) == \
                -(-(ref.tokens[op.node] + op.n) // ref.P) - len(ref.pages[op.node])
            tree.append_step(op.node, None, None, n_tokens=op.n)
            ref.append(op.node, op.n)
        else:
            tree.prune(op.node)
            ref.prune(op.node)
        if check_every_op:
            assert tree.free_pages() == ref.free_list()
            assert tree.stats() == ref.stats()


@pytest.mark.parametrize("seed", range(10))
def test_page_lists_and_free_list_bit_exact(seed):
    wl = sw.random_trace(300 + seed, n_ops=90, max_tokens=50, max_q_len=3)
    rng = np.random.default_rng(seed)
    n_pages = wl.peak_pages() + 5
    order = rng.permutation(n_pages).tolist() if seed % 2 else None
    tree, ref = host_tree(wl, n_pages, order), PageTableRef(n_pages, 16, order)
    replay_both(wl, tree, ref, check_every_op=True)
    for u in range(len(ref.parent)):
        if ref.alive[u]:
            assert tree.path_pages(u) == ref.path_pages(u)
            info = tree.node_info(u)
            assert info["parent"] == ref.parent[u] and info["n_tokens"] == ref.tokens[u]
            assert info["n_pages"] == len(ref.pages[u])
            assert info["n_live_children"] == sum(ref.alive[c] for c in ref.children[u])
        else:
            with pytest.raises(spex.SpexError) as e:
                tree.path_pages(u)
            assert e.value.name == "BAD_NODE"


PLAN_KEYS = ["leaf_indptr", "leaf_pages", "leaf_valid", "qt_limit", "group_node", "n_prefix_tasks",
             "n_partial_rows", "task_pg_begin", "task_pg_count", "task_qt_begin", "task_qt_count",
             "task_pbase", "task_flags", "pg_id", "pg_valid", "pg_pos", "qt_list", "part_indptr",
             "part_base", "part_hstride", "merge_qt"]


def assert_same_plan(tree, ref, wl, pc, sc):
    tree.set_tuning(pc, sc, 0, 0, 0)
    got = tree.plan_dump(wl.leaves, wl.q_lens)
    want = ref.plan(wl.leaves, wl.q_lens, wl.num_q_heads, wl.num_kv_heads,
                    got["prefix_chunk_pages"], got["suffix_chunk_pages"])
    if pc:
        assert got["prefix_chunk_pages"] == pc
    if sc:
        assert got["suffix_chunk_pages"] == sc
    for k in PLAN_KEYS:
        assert got[k] == want[k], k


@pytest.mark.parametrize("seed", range(8))
def test_plan_bit_exact_random_traces(seed):
    wl = sw.random_trace(400 + seed, n_ops=80, max_tokens=70, max_q_len=4,
                         heads=[(8, 2, 64), (6, 6, 32), (28, 4, 128)][seed % 3])
    n_pages = wl.peak_pages()
    order = np.random.default_rng(seed).permutation(n_pages).tolist()
    tree, ref = host_tree(wl, n_pages, order), PageTableRef(n_pages, 16, order)
    replay_both(wl, tree, ref)
    for pc, sc in ((0, 0), (1, 1), (2, 3), (1000, 1000)):
        assert_same_plan(tree, ref, wl, pc, sc)


@pytest.mark.parametrize("wl", [
    sw.tiny_tree(), sw.bfs_tot(n_queries=3), sw.mcts_skewed(n_queries=6),
    sw.spec_at_scale(n_queries=4), sw.tot_with_drafts(n_queries=3)], ids=lambda w: w.name)
def test_plan_bit_exact_config_shapes(wl):
    n_pages = wl.peak_pages()
    tree, ref = host_tree(wl, n_pages), PageTableRef(n_pages, 16)
    replay_both(wl, tree, ref)
    assert tree.stats() == ref.stats()
    for pc, sc in ((0, 0), (16, 8)):
        assert_same_plan(tree, ref, wl, pc, sc)


def test_full_size_config_4_plan_counts():
    wl = sw.spec_at_scale()
    tree = host_tree(wl, wl.peak_pages())
    ref = PageTableRef(wl.peak_pages(), 16)
    replay_both(wl, tree, ref)
    assert tree.stats() == (256 * 36, 176128, 0)
    pl = tree.plan_dump(wl.leaves, wl.q_lens)
    assert len(pl["pg_id"]) == wl.unique_kv_tokens() // 16 and len(set(pl["pg_id"])) == len(pl["pg_id"])
    assert pl["leaf_indptr"][-1] == wl.flat_kv_tokens() // 16
    want = ref.plan(wl.leaves, wl.q_lens, 64, 8, pl["prefix_chunk_pages"], pl["suffix_chunk_pages"])
    for k in PLAN_KEYS:
        assert pl[k] == want[k], k


def test_error_paths_leave_the_tree_unchanged():
    t = spex.SpexTree(8, 2, 64, 16, "bf16", "bf16", num_pages=4, host_only=True)
    (r,) = t.fork(-1, 1)
    t.append_step(r, None, None, n_tokens=20)                 # 2 pages
    a, b = t.fork(r, 2)
    before = (t.free_pages(), t.stats(), t.path_pages(a))
    with pytest.raises(spex.SpexError) as e:
        t.append_step(r, None, None, n_tokens=1)              # r has children
    assert e.value.name == "NOT_LEAF"
    with pytest.raises(spex.SpexError) as e:
        t.append_step(a, None, None, n_tokens=33)             # needs 3 pages, 2 free
    assert e.value.name == "OOM_PAGES"
    with pytest.raises(spex.SpexError) as e:
        t.fork(99, 1)
    assert e.value.name == "BAD_NODE"
    with pytest.raises(spex.SpexError) as e:
        t.plan_dump([a], [1 + 20 + 1])                         # more queries than path tokens
    assert e.value.name == "EMPTY_PATH"
    with pytest.raises(spex.SpexError) as e:
        t.plan_dump([a], [0])
    assert e.value.name == "INVALID_ARG"
    assert before == (t.free_pages(), t.stats(), t.path_pages(a))
    t.append_step(a, None, None, n_tokens=32)                 # exactly fits
    assert t.stats() == (3, 4, 0)
    t.prune(a)
    with pytest.raises(spex.SpexError) as e:
        t.prune(a)
    assert e.value.name == "BAD_NODE"
    t.prune(b)
    t.append_step(r, None, None, n_tokens=12)                 # childless again: fills page 2 of r
    assert t.node_info(r)["n_tokens"] == 32 and t.stats() == (1, 2, 2)
    t.prune(r)
    assert t.stats() == (0, 0, 4)
    with pytest.raises(spex.SpexError):
        spex.SpexTree(8, 3, 64, 16, "bf16", "bf16", num_pages=4, host_only=True)     # 8 % 3
    with pytest.raises(spex.SpexError):
        spex.SpexTree(8, 2, 64, 24, "bf16", "bf16", num_pages=4, host_only=True)     # page size
    with pytest.raises(spex.SpexError) as e:
        spex.SpexTree(8, 2, 64, 16, "f32", "bf16", num_pages=4, host_only=True)      # dtype pair
    assert e.value.name == "UNSUPPORTED"
    with pytest.raises(spex.SpexError):
        spex.SpexTree(8, 2, 64, 16, "bf16", "bf16", num_pages=4, host_only=True, free_order=[0, 1, 1, 3])


def test_plan_is_cached_until_the_tree_changes():
    wl = sw.bfs_tot(n_queries=1, prompt=32, step=16)
    t = host_tree(wl, wl.peak_pages() + 2)
    ref = PageTableRef(wl.peak_pages() + 2, 16)
    replay_both(wl, t, ref)
    p1 = t.plan_dump(wl.leaves, wl.q_lens)
    t.append_step(wl.leaves[0], None, None, n_tokens=1)
    ref.append(wl.leaves[0], 1)
    p2 = t.plan_dump(wl.leaves, wl.q_lens)
    assert p1["qt_limit"][0] + 1 == p2["qt_limit"][0]
    want = ref.plan(wl.leaves, wl.q_lens, wl.num_q_heads, wl.num_kv_heads,
                    p2["prefix_chunk_pages"], p2["suffix_chunk_pages"])
    for k in PLAN_KEYS:
        assert p2[k] == want[k], k


# ------------------------------------------------------------------ tree-walk lists
WALK_KEYS = ["available", "row_tiles", "waves", "row_blocks", "blocks", "qt", "items"]


def check_walk_lists(tree, ref, wl, row_tiles, waves=0):
    """Bit-exact against the reference model, and -- independently of both -- every row of every
    row block meets every page of its path exactly once, with the right positions and masks."""
    tree.set_tuning(0, 0, 0, row_tiles, waves)
    got = tree.walk_dump(wl.leaves, wl.q_lens, wl.draft_masks)
    want = ref.walk_plan(wl.leaves, wl.q_lens, wl.num_q_heads, wl.num_kv_heads, row_tiles, waves,
                         draft_masks=wl.draft_masks)
    for k in WALK_KEYS:
        assert got[k] == want[k], k
    return check_walk_coverage(got, ref, wl, row_tiles, waves)


def check_walk_coverage(got, ref, wl, row_tiles=0, waves=0, fresh=True):
    """The model-independent part: what the lists of `got` make every row read.  fresh=False: a
    plan that was patched after appends -- room may have been used up, and a block's flag bit 1
    is not re-derived."""
    G = wl.num_q_heads // wl.num_kv_heads
    q_lens = wl.q_lens if wl.q_lens is not None else [1] * len(wl.leaves)
    masks = wl.draft_masks                                       # the chain if none are given
    if masks is None:
        masks = [(2 << j) - 1 for ql in q_lens for j in range(ql)]
    if not got["available"]:
        # one query token does not fit a wavefront, or four row tiles were asked of the kernel that
        # splits the path (two wavefronts of rows)
        assert G > (16 * row_tiles if row_tiles else 64) or (waves == 2 and row_tiles == 4)
        return got
    C = 16 * got["row_tiles"]
    NW = got["waves"]
    assert NW in (2, 4, 8) and (waves == 0 or NW == waves)
    rbs = np.array(got["row_blocks"]).reshape(-1, 3 + 3 * NW)
    blocks = np.array(got["blocks"]).reshape(-1, 8)
    qt = np.array(got["qt"]).reshape(-1, 2)
    qoff = np.concatenate([[0], np.cumsum(q_lens)])
    tok_owner = np.repeat(np.arange(len(wl.leaves)), q_lens)        # query token -> request
    seen_tokens = []
    used_blocks = np.zeros(len(blocks), dtype=bool)
    rbs_of_page = {}                                              # page -> row blocks that list it
    def spans_of(rb):
        """(first block, end, wavefront or None for the shared blocks), and the unused room"""
        first, n_sh = rb[1], rb[2]
        out, gaps = [(first, first + n_sh, None)], []
        b0 = first + n_sh
        for w in range(NW):
            count, room = int(rb[3 + w]) & 0xffff, int(rb[3 + w]) >> 16
            assert room >= count
            out.append((b0, b0 + count, w))
            gaps.append((b0 + count, b0 + room))
            b0 += room
        return out, gaps

    childless = {u for u in set(wl.leaves) if not ref.has_live_children(u)}
    for bi, rb in enumerate(rbs):
        for a, b, _ in spans_of(rb)[0]:
            for blk in blocks[a:b]:
                for pg in {int(blk[0]), int(blk[2])}:
                    rbs_of_page.setdefault(pg, set()).add(bi)
    for rb in rbs:
        spans, gaps = spans_of(rb)
        for a, b in gaps:                                         # unused room: all-zero records
            assert not blocks[a:b].any()
            used_blocks[a:b] = True
        if fresh:                                                 # flag bit 1: shared between row blocks
            for a, b, _ in spans:
                for blk in blocks[a:b]:
                    assert bool(blk[5] & 2) == (len(rbs_of_page[int(blk[0])]) > 1)
        first, n_sh = rb[1], rb[2]
        qt_first, qt_count = rb[3 + NW:3 + 2 * NW], rb[3 + 2 * NW:3 + 3 * NW]
        # rows of the row block: row -> (query token, limit)
        row_tok = {}
        for w in range(NW):
            for e in range(qt_count[w]):
                t, lim = qt[qt_first[w] + e]
                assert lim == ref_limit(ref, wl, tok_owner[t], t - qoff[tok_owner[t]], q_lens)
                j = t - qoff[tok_owner[t]]
                hidden = [lim - 1 - j + k for k in range(q_lens[tok_owner[t]]) if not (masks[t] >> k) & 1]
                for hh in range(G):
                    row_tok[w * C + e * G + hh] = (t, hidden)
                seen_tokens.append(t)
            assert qt_count[w] * G <= C
        if fresh:        # room: two records per requested childless node that is private to the wavefront
            for (a, b, w), (ga, gb) in zip(spans[1:], gaps):
                own_pages = {int(blk[0]) for blk in blocks[a:b]}
                nodes_here = {u for u in childless if ref.pages[u] and ref.pages[u][0] in own_pages
                              and any(wl.leaves[tok_owner[qt[qt_first[w] + e][0]]] == u for e in range(qt_count[w]))}
                assert gb - ga == 2 * len(nodes_here), (w, gb - ga, nodes_here)
        pages_of_row = {r: [] for r in row_tok}
        for a, b, wave in spans:
            for blk in blocks[a:b]:
                lo, hi = blk[4] & 0xffff, blk[4] >> 16
                assert lo < hi
                if wave is None:
                    assert lo // C != (hi - 1) // C                 # really shared by >= 2 wavefronts
                else:
                    assert lo // C == wave and (hi - 1) // C == wave
                entries = [(blk[0], blk[1] >> 7, blk[1] & 127)]
                if blk[3]:
                    entries.append((blk[2], blk[3] >> 7, blk[3] & 127))
                    assert (blk[1] & 127) == 16
                start, end = entries[0][1], entries[-1][1] + entries[-1][2]
                need_mask = len(entries) == 1 or any(v != 16 for _, _, v in entries)
                for r, (t, hidden) in row_tok.items():
                    if lo <= r < hi:
                        pages_of_row[r] += entries
                        need_mask = need_mask or any(start <= h < end for h in hidden)
                assert (blk[5] & 1) or not need_mask               # a needed mask is never dropped
            used_blocks[a:b] = True
        for r, (t, _) in row_tok.items():
            pages, valid = ref.path_pages(wl.leaves[tok_owner[t]])
            pos = np.concatenate([[0], np.cumsum(valid)])[:-1]
            want_entries = sorted((p, int(s), v) for p, s, v in zip(pages, pos, valid) if v > 0)
            assert sorted(pages_of_row[r]) == want_entries, (r, t)
    assert sorted(seen_tokens) == list(range(qoff[-1]))            # every query token in one row block
    assert used_blocks.all()
    S = 16 if NW <= 4 else 32
    items = np.array(got["items"]).reshape(-1, S)
    real = items[items[:, S - 1] >= 0]
    assert len(real) == len(rbs) * wl.num_kv_heads
    for g in range(wl.num_kv_heads):
        assert sorted(real[real[:, 0] == g][:, S - 1].tolist()) == list(range(len(rbs)))
    for it in real:
        assert it[1:3 + 3 * NW].tolist() == rbs[it[S - 1]][1:].tolist()
        assert (it[3 + 3 * NW:S - 1] == 0).all()
    assert (items[items[:, S - 1] < 0][:, 1:S - 1] == 0).all()
    return got


def ref_limit(ref, wl, req, j, q_lens):
    T = sum(ref.tokens[w] for w in ref.path(wl.leaves[req]))
    return T - q_lens[req] + 1 + j


@pytest.mark.parametrize("seed", range(8))
def test_walk_lists_random_traces(seed):
    wl = sw.random_trace(500 + seed, n_ops=80, max_tokens=70, max_q_len=[1, 4, 9][seed % 3],
                         heads=[(8, 2, 64), (6, 6, 32), (28, 4, 128), (8, 1, 128)][seed % 4])
    n_pages = wl.peak_pages()
    order = np.random.default_rng(seed).permutation(n_pages).tolist()
    tree, ref = host_tree(wl, n_pages, order), PageTableRef(n_pages, 16, order)
    replay_both(wl, tree, ref)
    for rt in (0, 1, 2, 4):
        for nw in (0, 4, 8):
            check_walk_lists(tree, ref, wl, rt, nw)


@pytest.mark.parametrize("wl", [
    sw.bfs_tot(n_queries=3), sw.mcts_skewed(n_queries=6), sw.spec_at_scale(n_queries=4),
    sw.tot_with_drafts(n_queries=3),
    sw.bfs_tot(n_queries=1, prompt=9000, step=1100, width=4, keep=2, depth=2, heads=(8, 2, 128)),   # few long paths
    sw.mcts_skewed(n_queries=2, prompt=(3000, 6000), step=(300, 700), max_leaves=6)],
    ids=lambda w: f"{w.name}_{w.n_trees}_{len(w.leaves)}")
def test_walk_lists_config_shapes(wl):
    n_pages = wl.peak_pages()
    tree, ref = host_tree(wl, n_pages), PageTableRef(n_pages, 16)
    replay_both(wl, tree, ref)
    got = check_walk_lists(tree, ref, wl, 0)
    assert got["available"] == 1
    assert got["waves"] == 4
    for rt in (1, 2, 4):
        for nw in (2, 4, 8):
            check_walk_lists(tree, ref, wl, rt, nw)


@pytest.mark.parametrize("seed", range(4))
def test_walk_lists_with_draft_token_trees(seed):
    """Sec. 6.5 token trees: the mask flag of a block follows the first draft some query does not
    see; everything else is as for the chain."""
    if seed < 3:
        wl = sw.with_draft_trees(sw.random_trace(520 + seed, n_ops=70, max_tokens=60, max_q_len=[4, 8, 16][seed],
                                                 heads=[(8, 2, 64), (4, 4, 128), (4, 2, 64)][seed]))
    else:
        wl = sw.tot_with_drafts(n_queries=2, prompt=70, step=33, drafts=6, token_trees=True)
    assert any(m != (2 << j) - 1 for ql, o in zip(wl.q_lens, np.cumsum([0] + wl.q_lens[:-1]))
               for j, m in enumerate(wl.draft_masks[o:o + ql]))
    n_pages = wl.peak_pages()
    tree, ref = host_tree(wl, n_pages), PageTableRef(n_pages, 16)
    replay_both(wl, tree, ref)
    for rt in (0, 1, 2):
        check_walk_lists(tree, ref, wl, rt, 4)
    # the chain written as masks gives the lists of the call without masks
    chain = [(2 << j) - 1 for ql in wl.q_lens for j in range(ql)]
    tree.set_tuning(0, 0, 0, 0, 0)
    a = tree.walk_dump(wl.leaves, wl.q_lens, chain)
    b = tree.walk_dump(wl.leaves, wl.q_lens)
    assert b["plan_state"] == 1                                  # masks are part of the cached request
    for k in WALK_KEYS:
        assert a[k] == b[k], k
    assert tree.walk_dump(wl.leaves, wl.q_lens)["plan_state"] == 0


def test_draft_mask_errors():
    t = spex.SpexTree(8, 2, 64, 16, "bf16", "bf16", num_pages=8, host_only=True)
    (r,) = t.fork(-1, 1)
    t.append_step(r, None, None, n_tokens=40)
    with pytest.raises(spex.SpexError) as e:
        t.walk_dump([r], [3], [1, 3, 8])                          # bit 3 with 3 drafts
    assert e.value.name == "INVALID_ARG"
    with pytest.raises(spex.SpexError) as e:
        t.walk_dump([r], [33], [1] * 33)                          # more than 32 drafts
    assert e.value.name == "INVALID_ARG"
    with pytest.raises(spex.SpexError) as e:
        t.walk_dump([r], None, [1])                               # masks need q_lens
    assert e.value.name == "INVALID_ARG"
    with pytest.raises(spex.SpexError) as e:
        t.walk_dump([r], [40], None)                              # chain of 40 is fine without masks ..
        t.walk_dump([r], [41], None)                              # .. 41 queries on 40 tokens are not
    assert e.value.name == "EMPTY_PATH"
    (s,) = t.fork(-1, 1)
    t.append_step(s, None, None, n_tokens=3)
    with pytest.raises(spex.SpexError) as e:
        t.walk_dump([s], [3], [1, 0, 5])                          # query 1 sees nothing at all
    assert e.value.name == "EMPTY_PATH"
    assert t.walk_dump([s], [3], [1, 2, 5])["available"] == 1
    assert t.walk_dump([r, s], [2, 3], [0, 0, 1, 2, 5])["available"] == 1   # r's drafts still see its prefix


def test_wide_requests_are_cut_into_pieces_of_query_tokens():
    wl = sw.random_trace(77, n_ops=30, max_tokens=90, max_q_len=9, heads=(16, 2, 64))   # up to 72 rows
    tree, ref = host_tree(wl, wl.peak_pages()), PageTableRef(wl.peak_pages(), 16)
    replay_both(wl, tree, ref)
    assert max(wl.q_lens) * 8 > 64
    got = check_walk_lists(tree, ref, wl, 0)
    assert got["available"] == 1 and got["row_tiles"] == 2       # 4 query tokens of 8 rows per wavefront
    for rt in (1, 2, 4):
        for nw in (2, 4, 8):
            assert check_walk_lists(tree, ref, wl, rt, nw)["available"] == (0 if (rt, nw) == (4, 2) else 1)
    # 9 queries: three pieces of three; the pieces' entries follow each other in qt
    qt = np.array(got["qt"]).reshape(-1, 2)[:, 0]
    qoff = np.concatenate([[0], np.cumsum(wl.q_lens)])
    for i, ql in enumerate(wl.q_lens):
        at = int(np.flatnonzero(qt == qoff[i])[0])
        assert qt[at:at + ql].tolist() == list(range(qoff[i], qoff[i] + ql))


def test_walk_lists_not_available_when_one_query_token_is_wider_than_a_wavefront():
    wl = sw.random_trace(78, n_ops=20, max_tokens=50, max_q_len=2, heads=(40, 1, 64))   # G = 40
    tree, ref = host_tree(wl, wl.peak_pages()), PageTableRef(wl.peak_pages(), 16)
    replay_both(wl, tree, ref)
    for rt, avail in ((0, 1), (4, 1), (2, 0), (1, 0)):
        got = check_walk_lists(tree, ref, wl, rt)
        assert got["available"] == avail and (avail or got["items"] == [])
    wl = sw.random_trace(79, n_ops=20, max_tokens=50, heads=(80, 1, 64))                # G = 80
    tree, ref = host_tree(wl, wl.peak_pages()), PageTableRef(wl.peak_pages(), 16)
    replay_both(wl, tree, ref)
    assert check_walk_lists(tree, ref, wl, 0)["available"] == 0


# ------------------------------------------------------------------ length patches
def grow_and_compare(wl, n_steps, seed, walk_only=False, max_run=3, row_tiles=0, waves=0):
    """Append tokens to requested leaves step by step.  The library patches its cached lists when
    it can: always when no page is started; when pages are started, if the tree-walk lists are
    the plan's only lists and the room behind the grown node's wavefront is not used up.  A second
    tree that replays everything and plans afresh must give the same lists as a fresh plan, and as
    a plan patched without page starts, except that a patched plan may keep mask flags a fresh
    plan no longer needs; a plan patched with page starts is checked for what it makes every row
    read (its new blocks sit in the room, not where a fresh plan puts them).
    Returns (patches without page start, fresh plans, patches with page starts)."""
    n_pages = wl.peak_pages() + (8 + n_steps * max_run // 16) * len(wl.leaves) + 8
    tree, ref = host_tree(wl, n_pages), PageTableRef(n_pages, 16)
    replay_both(wl, tree, ref)
    rng = np.random.default_rng(seed)
    childless = [u for u in sorted(set(wl.leaves)) if not ref.has_live_children(u)]
    masks = wl.draft_masks          # with masks only the tree-walk lists are compared: the
    split = masks is None and not walk_only     # split lists' dump takes no masks and would plan afresh
    tree.set_tuning(0, 0, 0, row_tiles, waves)
    if split:
        tree.plan_dump(wl.leaves, wl.q_lens)
    tree.walk_dump(wl.leaves, wl.q_lens, masks)
    patched_seen = fresh_seen = page_patches = 0
    moved = False                   # blocks were started by a patch since the last fresh plan
    for step in range(n_steps):
        grow = [u for u in childless if rng.random() < 0.7]
        started_page = False
        for u in grow:
            n = int(rng.integers(1, max_run + 1))
            started_page |= tree.append_new_pages(u, n) > 0
            tree.append_step(u, None, None, n_tokens=n)
            ref.append(u, n)
        got_walk = tree.walk_dump(wl.leaves, wl.q_lens, masks)
        state = got_walk["plan_state"]
        if grow:
            if split or not got_walk["available"]:
                assert state == (1 if started_page else 2), step
            else:
                assert state in ((1, 2) if started_page else (2,)), step
        if grow:
            patched_seen += state == 2 and not started_page
            fresh_seen += state == 1
        if state == 1:
            moved = False
        elif started_page and grow:
            moved = True
            page_patches += 1
        if moved:
            check_walk_coverage(got_walk, ref, wl, row_tiles, waves, fresh=False)
            continue
        want_walk = ref.walk_plan(wl.leaves, wl.q_lens, wl.num_q_heads, wl.num_kv_heads, row_tiles, waves,
                                  draft_masks=masks)
        got_split = want_split = {}
        if split:
            got_split = tree.plan_dump(wl.leaves, wl.q_lens)
            want_split = ref.plan(wl.leaves, wl.q_lens, wl.num_q_heads, wl.num_kv_heads,
                                  got_split["prefix_chunk_pages"], got_split["suffix_chunk_pages"])
        for k in (PLAN_KEYS if split else []):
            if k == "task_flags":
                for a, b in zip(got_split[k], want_split[k]):
                    assert a & 2 == b & 2 and (a & 1) >= (b & 1)
            else:
                assert got_split[k] == want_split[k], (step, k)
        for k in WALK_KEYS:
            if k == "blocks":
                a, b = np.array(got_walk[k]).reshape(-1, 8), np.array(want_walk[k]).reshape(-1, 8)
                assert np.array_equal(a[:, :5], b[:, :5]) and np.array_equal(a[:, 5] & 2, b[:, 5] & 2)
                assert np.all((a[:, 5] & 1) >= (b[:, 5] & 1))
            else:
                assert got_walk[k] == want_walk[k], (step, k)
    return patched_seen, fresh_seen, page_patches


GROW_WORKLOADS = [
    sw.bfs_tot(n_queries=2, prompt=40, step=19), sw.tot_with_drafts(n_queries=2, prompt=50, step=21),
    sw.mcts_skewed(n_queries=4, prompt=(30, 90), step=(5, 40), max_leaves=12),
    sw.random_trace(640, n_ops=60, max_tokens=40, max_q_len=3, heads=(8, 2, 64)),
    sw.with_draft_trees(sw.random_trace(641, n_ops=14, max_tokens=40, max_q_len=5, heads=(8, 2, 64))),
    sw.random_trace(642, n_ops=16, max_tokens=40, max_q_len=9, heads=(16, 2, 64))]      # requests cut into pieces


@pytest.mark.parametrize("wl", GROW_WORKLOADS, ids=lambda w: w.name)
def test_length_patches_match_a_fresh_plan(wl):
    patched, fresh, _ = grow_and_compare(wl, 24, 5)
    assert patched > 3 and (fresh > 3 or wl.draft_masks is not None)    # both paths were taken


@pytest.mark.parametrize("wl", GROW_WORKLOADS[:4] + [sw.random_trace(643, n_ops=40, max_tokens=50, max_q_len=1, heads=(28, 4, 128))],
                         ids=lambda w: w.name)
def test_patches_that_start_pages(wl):
    """Tree-walk lists alone: started pages go into the last block's free half or into the room
    of the node's wavefront, until the room is used up and the plan is made afresh."""
    patched, fresh, page_patches = grow_and_compare(wl, 90, 9, walk_only=True)
    assert page_patches > 10 and fresh > 0 and patched > 3


@pytest.mark.parametrize("row_tiles,waves", [(2, 4), (1, 8), (4, 8), (2, 2), (1, 2)])
def test_patches_that_start_pages_other_row_block_shapes(row_tiles, waves):
    wl = sw.mcts_skewed(n_queries=4, prompt=(30, 90), step=(5, 40), max_leaves=12)
    patched, fresh, page_patches = grow_and_compare(wl, 90, 23, walk_only=True, row_tiles=row_tiles, waves=waves)
    assert page_patches > 10 and fresh > 0 and patched > 3


@pytest.mark.parametrize("wl", GROW_WORKLOADS[4:], ids=lambda w: w.name)
def test_started_pages_of_nodes_that_several_wavefronts_share(wl):
    """Draft token trees, and requests cut into pieces: a grown node whose rows lie in several
    wavefronts sits among the shared blocks, which have no room -- its started page can still become
    page b of its last block, otherwise the plan is made afresh.  Either way the lists must cover
    every row's path."""
    patched, fresh, page_patches = grow_and_compare(wl, 60, 17, walk_only=True)
    assert patched > 3 and fresh > 0 and page_patches > 0


def test_started_page_of_a_node_requested_twice_plans_afresh():
    wl = sw.bfs_tot(n_queries=1, prompt=40, step=19)
    n_pages = wl.peak_pages() + 16
    tree, ref = host_tree(wl, n_pages), PageTableRef(n_pages, 16)
    replay_both(wl, tree, ref)
    leaves = list(wl.leaves) + [wl.leaves[0]]                  # the first branch asked for twice
    assert tree.walk_dump(leaves, None)["plan_state"] == 1
    u = wl.leaves[0]
    seen = set()
    for _ in range(40):
        started = tree.append_new_pages(u, 1) > 0
        tree.append_step(u, None, None, n_tokens=1)
        ref.append(u, 1)
        got = tree.walk_dump(leaves, None)
        assert got["plan_state"] == (1 if started else 2)
        seen.add(got["plan_state"])
        want = ref.walk_plan(leaves, None, wl.num_q_heads, wl.num_kv_heads)
        for k in ("row_blocks", "qt", "items"):
            assert got[k] == want[k], k
    assert seen == {1, 2}


@pytest.mark.parametrize("wl", GROW_WORKLOADS[:3], ids=lambda w: w.name)
def test_patches_that_start_several_pages_at_once(wl):
    """Runs of up to 45 tokens: one append can fill the last block's free half, open a block in the
    room and fill that block's second half as well."""
    _, fresh, page_patches = grow_and_compare(wl, 30, 13, walk_only=True, max_run=45)
    assert page_patches > 5 and fresh > 0


# ------------------------------------------------------------------ one token per node
def test_append_tokens_matches_single_appends_and_is_all_or_nothing():
    wl = sw.bfs_tot(n_queries=2, prompt=40, step=15)
    n_pages = wl.peak_pages() + 3 * len(wl.leaves)
    order = np.random.default_rng(4).permutation(n_pages).tolist()
    tree, ref = host_tree(wl, n_pages, order), PageTableRef(n_pages, 16, order)
    replay_both(wl, tree, ref)
    leaves = list(wl.leaves)
    for it in range(20):                                      # crosses page boundaries
        nodes = leaves[::2] if it % 3 == 0 else leaves
        tree.append_tokens(nodes, None, None)
        for u in nodes:
            ref.append(u, 1)                                   # same page order as one call per node
        assert tree.free_pages() == ref.free_list() and tree.stats() == ref.stats()
        for u in leaves[:5]:
            assert tree.path_pages(u) == ref.path_pages(u)
    before = (tree.free_pages(), tree.stats(), [tree.node_info(u)["n_tokens"] for u in leaves])
    root = ref.path(leaves[0])[0]
    for bad, name in (([leaves[0], 10 ** 6], "BAD_NODE"), ([leaves[0], leaves[1], leaves[0]], "INVALID_ARG"),
                      ([leaves[1], root], "NOT_LEAF")):
        with pytest.raises(spex.SpexError) as e:
            tree.append_tokens(bad, None, None)
        assert e.value.name == name
        assert before == (tree.free_pages(), tree.stats(), [tree.node_info(u)["n_tokens"] for u in leaves])
    # too few pages for all: nothing happens to any of them
    small = spex.SpexTree(8, 2, 64, 16, "bf16", "bf16", num_pages=3, host_only=True)
    (r,) = small.fork(-1, 1)
    small.append_step(r, None, None, n_tokens=16)
    kids = small.fork(r, 3)
    with pytest.raises(spex.SpexError) as e:
        small.append_tokens(kids, None, None)                 # needs 3 pages, 2 free
    assert e.value.name == "OOM_PAGES" and small.stats() == (4, 1, 2)
    small.append_tokens(kids[:2], None, None)
    assert small.stats() == (4, 3, 0)


def test_quantising_append_is_for_fp8_pools_only():
    t = spex.SpexTree(4, 2, 96, 16, "bf16", "fp8_e4m3", num_pages=4, host_only=True)
    (r,) = t.fork(-1, 1)
    t.append_tokens([r], None, None, quantize=True)            # page table only
    assert t.node_info(r)["n_tokens"] == 1
    b = spex.SpexTree(4, 2, 64, 16, "bf16", "bf16", num_pages=4, host_only=True)
    (r,) = b.fork(-1, 1)
    with pytest.raises(spex.SpexError) as e:
        b.append_tokens([r], None, None, quantize=True)
    assert e.value.name == "UNSUPPORTED" and b.node_info(r)["n_tokens"] == 0
