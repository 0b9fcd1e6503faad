"""Reference model of the tree page table and of the per-launch plan -- TEST INFRASTRUCTURE.

A dictionary-and-list model, written independently of the C++ library, of the
integer side of the hot path: which physical pages hold which node's tokens,
what pruning gives back, and how a set of requested nodes is flattened into
root-to-node page lists, shared-prefix groups, private suffixes, split chunks
and the partial-result slots the merge step reads.  Page lists, free lists and
plans must match the library bit for bit, so the rules are written out here.

Tree (paper Sec. 2.1: a node is the state reached by one step, i.e. a run of
tokens; Alg. 2: children are added for primary and speculative expansions;
Sec. 4.2: a mis-speculated BFS branch is terminated at once):
  * node ids are dense, follow creation order and are never reused;
  * a node's tokens fill pages of `page_size` slots in order; only its last page
    may be partial; a child never continues its parent's last page, so a page
    belongs to exactly one node;
  * tokens may be appended only to a node without live children.

Allocator: a stack.  Initially page free_order[0] is on top, then free_order[1]
and so on (ascending ids if no order is given).  An append pops one page at a
time in token order; an append that does not fit changes nothing.  Prune visits
the subtree in pre-order (children in creation order) and pushes each visited
node's pages in run order.

Plan for requested nodes leaves[0..L) with q_lens (caller order):
  * query tokens are numbered 0..NQ) leaf-major; query token (leaf, i) sees
    limit = T - q_len + 1 + i path positions;
  * live[u] = number of requested nodes in u's subtree (u included);
  * a GROUP is a node on a requested path with live >= 2 and at least one token;
    groups are listed by ascending node id; a group's rows are the query tokens
    of all requested nodes below it, in caller order;
  * the SUFFIX of requested node l is the maximal tail of its path with
    live == 1, root side first, empty nodes skipped; it may be empty;
  * a segment (group or suffix) of n pages is cut into c = ceil(n / chunk_pages)
    chunks, chunk j covering pages [j*n // c, (j+1)*n // c);
  * TASKS: one per chunk, all group chunks first (group order, chunk order), then
    suffix chunks (caller order, chunk order).  A task owns
    rows * Hkv partial slots starting at pbase (running sum in task order), where
    rows = (number of query tokens of its segment) * (Hq / Hkv); the slot of
    (kv head g, local query token r, head-in-group hh) is
    pbase + g * rows + r * G + hh;
  * a task is flagged MASKED (flag bit 0) if one of its pages is partial or if
    some row's limit is smaller than the path position that follows its last token;
    a suffix task that is the only chunk of its suffix is flagged FINAL (flag bit 1):
    it is the last piece of its rows, so the kernel that computes it can combine it
    with the rows' other pieces and write the output itself;
  * merge_qt lists, ascending, the query tokens that still need the separate merge
    step: those of requested nodes whose suffix is empty or cut into several chunks;
  * the merge list of a query token holds, in task order, for every task that
    has it as a row: base = pbase + r * G and hstride = rows.

Tree-walk lists (second kernel set: one workgroup carries a block of query rows
from the root to the requested nodes).  With G = Hq / Hkv, request i has
q_len_i * G rows and C = 16 * row_tiles rows fit one wavefront:
  * row_tiles is the value asked for (1, 2, 4) or, if 0: 1 if no request has
    more than 16 rows (raised to 2 when some root has more than 64 rows below
    it and sum over roots of ceil(rows / 128), times Hkv, is at least 512), 2 if
    none has more than 32, else 2 (4 if G > 32); no lists if G > C;
  * roots in order of first appearance; a root's requests sorted by path (node
    ids root first, lexicographic, a proper prefix first; ties in request
    order), so the requests below any node are consecutive;
  * a request with more than cap = C // G query tokens is cut into
    ceil(q_len / cap) pieces of consecutive query tokens, the first
    q_len mod pieces of them one token longer than the rest; "request" below
    means such a piece;
  * a row block has NW wavefronts of rows: the value asked for (2, 4, 8); if 0: 8 if there are no
    draft masks, NTW <= 2, no request has more than C rows, some root has more than 4 C rows and
    sum over roots of ceil(rows / (8 C)), times Hkv, is at least 1024; else 4;
  * a request joins the current wavefront while its rows fit, else starts the
    next; wavefront NW or a new root starts a new row block; `qt` lists
    (query token, limit) of the requests in this order; the row of a request in
    its row block is wavefront * C + rows before it in the wavefront;
  * the nodes of a row block are the nodes with tokens on its requests' paths in
    order of first encounter, with row range [first row of the first request
    through it, last row + 1 of the last one) and minlim = min over those requests
    of the first path position some query of the request does not see: T - q_len
    + 1 for the causal chain; with draft masks (query j sees everything before
    the q_len drafts and draft k iff bit k of mask j is set) T - q_len + the
    number of leading drafts that all of the request's queries see; a node whose
    range touches two wavefronts is shared, else private to wavefront lo // C;
  * blocks of a row block: shared nodes first, then the private nodes of
    wavefront 0..NW-1, each wavefront's blocks followed by room for blocks that
    later appends start: two all-zero records per private node of the wavefront
    that a request of the row block asks for and that has no live children; the
    row block and the work items hold count | (count + room) << 16 per
    wavefront (no lists if that exceeds 16 bits); a node's pages two at a time;
    record (page a, pos_a << 7 |
    valid_a, page b or a again, pos_b << 7 | valid_b or 0, lo | hi << 16, flag, 0,
    0); flag bit 0 = a page partial or missing, or minlim < position after the
    block; flag bit 1 = the node lies on paths of more than one row block;
  * launch order: roots by descending block count (stable); lanes = 8 // Hkv for
    Hkv in (1, 2, 4) else 1; each root goes to the lane with the fewest blocks so
    far; round r emits for every lane its r-th row block (padding if it ran out
    and lanes > 1), each for kv head 0..Hkv-1.
"""

from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

NO_NODE = -1


class OutOfPages(Exception):
    pass


class PageTableRef:
    def __init__(self, num_pages: int, page_size: int = 16,
                 free_order: Optional[Sequence[int]] = None):
        self.P = page_size
        self.num_pages = num_pages
        order = list(range(num_pages)) if free_order is None else list(free_order)
        assert sorted(order) == list(range(num_pages))
        self.free: List[int] = order[::-1]            # stack: top is the END of the list
        self.parent: List[int] = []
        self.children: List[List[int]] = []
        self.alive: List[bool] = []
        self.tokens: List[int] = []
        self.pages: List[List[int]] = []

    # ---------------------------------------------------------------- mutation
    def _check(self, u: int) -> None:
        if not (0 <= u < len(self.parent)) or not self.alive[u]:
            raise KeyError(u)

    def fork(self, parent: int, n: int) -> List[int]:
        if parent != NO_NODE:
            self._check(parent)
        ids = []
        for _ in range(n):
            u = len(self.parent)
            self.parent.append(parent)
            self.children.append([])
            self.alive.append(True)
            self.tokens.append(0)
            self.pages.append([])
            if parent != NO_NODE:
                self.children[parent].append(u)
            ids.append(u)
        return ids

    def has_live_children(self, u: int) -> bool:
        return any(self.alive[c] for c in self.children[u])

    def append(self, u: int, n_tokens: int) -> List[int]:
        """Returns the pages newly started by this append."""
        self._check(u)
        if self.has_live_children(u):
            raise ValueError("not a leaf")
        need = -(-(self.tokens[u] + n_tokens) // self.P) - len(self.pages[u])
        if need > len(self.free):
            raise OutOfPages()
        new = [self.free.pop() for _ in range(need)]
        self.pages[u].extend(new)
        self.tokens[u] += n_tokens
        return new

    def prune(self, u: int) -> None:
        self._check(u)
        stack = [u]
        while stack:                                   # pre-order, children in creation order
            w = stack.pop()
            if not self.alive[w]:
                continue
            self.alive[w] = False
            for p in self.pages[w]:
                self.free.append(p)
            self.pages[w] = []
            stack.extend(reversed(self.children[w]))

    # ---------------------------------------------------------------- queries
    def stats(self):
        live = sum(self.alive)
        used = sum(len(p) for p in self.pages)
        return live, used, len(self.free)

    def free_list(self) -> List[int]:
        """Free pages, next page to be handed out first."""
        return self.free[::-1]

    def path(self, u: int) -> List[int]:
        self._check(u)
        p = []
        while u != NO_NODE:
            p.append(u)
            u = self.parent[u]
        return p[::-1]

    def node_page_valid(self, u: int):
        n = self.tokens[u]
        return [min(self.P, n - i * self.P) for i in range(len(self.pages[u]))]

    def path_pages(self, u: int):
        pages, valid = [], []
        for w in self.path(u):
            pages.extend(self.pages[w])
            valid.extend(self.node_page_valid(w))
        return pages, valid

    # ---------------------------------------------------------------- the plan
    def plan(self, leaves: Sequence[int], q_lens: Optional[Sequence[int]],
             num_q_heads: int, num_kv_heads: int,
             prefix_chunk_pages: int, suffix_chunk_pages: int) -> Dict[str, list]:
        L = len(leaves)
        q_lens = [1] * L if q_lens is None else list(q_lens)
        G = num_q_heads // num_kv_heads
        P = self.P
        paths = [self.path(u) for u in leaves]

        # root-to-node CSR
        leaf_indptr, leaf_pages, leaf_valid = [0], [], []
        for u in leaves:
            pg, va = self.path_pages(u)
            leaf_pages += pg
            leaf_valid += va
            leaf_indptr.append(len(leaf_pages))

        # query tokens and their visible lengths
        qoff, qt_limit = [], []
        for path, ql in zip(paths, q_lens):
            T = sum(self.tokens[w] for w in path)
            if ql < 1 or ql > T:
                raise ValueError("empty path or q_len > path length")
            qoff.append(len(qt_limit))
            qt_limit += [T - ql + 1 + i for i in range(ql)]
        NQ = len(qt_limit)

        live: Dict[int, int] = {}
        for path in paths:
            for w in path:
                live[w] = live.get(w, 0) + 1

        # path position of each node's first token (same for every path through it)
        pos0: Dict[int, int] = {}
        for path in paths:
            t = 0
            for w in path:
                pos0[w] = t
                t += self.tokens[w]

        group_nodes = sorted(w for w in live if live[w] >= 2 and self.tokens[w] > 0)
        gindex = {w: i for i, w in enumerate(group_nodes)}
        group_rows: List[List[int]] = [[] for _ in group_nodes]
        for li, (path, ql) in enumerate(zip(paths, q_lens)):
            for w in path:
                if w in gindex:
                    group_rows[gindex[w]] += list(range(qoff[li], qoff[li] + ql))

        qt_list: List[int] = []
        group_qt_begin = []
        for rows in group_rows:
            group_qt_begin.append(len(qt_list))
            qt_list += rows
        n_group_qt = len(qt_list)
        qt_list += list(range(NQ))

        def segment_entries(nodes):
            ids, valid, pos = [], [], []
            for w in nodes:
                va = self.node_page_valid(w)
                t = pos0[w]
                for p, v in zip(self.pages[w], va):
                    ids.append(p)
                    valid.append(v)
                    pos.append(t)
                    t += v
            return ids, valid, pos

        def cut(n, chunk):
            c = -(-n // chunk)
            return [(j * n // c, (j + 1) * n // c) for j in range(c)]

        tasks = dict(pg_begin=[], pg_count=[], qt_begin=[], qt_count=[], pbase=[], flags=[])
        pg_id, pg_valid, pg_pos = [], [], []
        parts: List[List[tuple]] = [[] for _ in range(NQ)]
        pbase = 0

        def emit(ids, valid, pos, chunk_pages, qt_begin, qt_count, suffix=False):
            nonlocal pbase
            rows = qt_count * G
            min_limit = min(qt_limit[qt_list[qt_begin + r]] for r in range(qt_count))
            pieces = cut(len(ids), chunk_pages)
            final = suffix and len(pieces) == 1
            for a, b in pieces:
                end_pos = pos[b - 1] + valid[b - 1]
                masked = any(v != P for v in valid[a:b]) or min_limit < end_pos
                tasks["pg_begin"].append(len(pg_id))
                tasks["pg_count"].append(b - a)
                tasks["qt_begin"].append(qt_begin)
                tasks["qt_count"].append(qt_count)
                tasks["pbase"].append(pbase)
                tasks["flags"].append((1 if masked else 0) | (2 if final else 0))
                pg_id.extend(ids[a:b])
                pg_valid.extend(valid[a:b])
                pg_pos.extend(pos[a:b])
                for r in range(qt_count):
                    parts[qt_list[qt_begin + r]].append((pbase + r * G, rows))
                pbase += rows * num_kv_heads
            return final

        for gi, w in enumerate(group_nodes):
            ids, valid, pos = segment_entries([w])
            emit(ids, valid, pos, prefix_chunk_pages, group_qt_begin[gi], len(group_rows[gi]))
        n_prefix_tasks = len(tasks["pbase"])
        merge_qt: List[int] = []
        for li, (path, ql) in enumerate(zip(paths, q_lens)):
            tail = []
            for w in reversed(path):
                if live[w] != 1:
                    break
                tail.append(w)
            ids, valid, pos = segment_entries(tail[::-1])
            if ids:
                final = emit(ids, valid, pos, suffix_chunk_pages, n_group_qt + qoff[li], ql, True)
            else:
                final = False
            if not final:
                merge_qt += list(range(qoff[li], qoff[li] + ql))

        part_indptr, part_base, part_hstride = [0], [], []
        for lst in parts:
            for b, h in lst:
                part_base.append(b)
                part_hstride.append(h)
            part_indptr.append(len(part_base))

        return dict(
            leaf_indptr=leaf_indptr, leaf_pages=leaf_pages, leaf_valid=leaf_valid,
            qt_limit=qt_limit, group_node=group_nodes,
            n_prefix_tasks=n_prefix_tasks, n_partial_rows=pbase,
            task_pg_begin=tasks["pg_begin"], task_pg_count=tasks["pg_count"],
            task_qt_begin=tasks["qt_begin"], task_qt_count=tasks["qt_count"],
            task_pbase=tasks["pbase"], task_flags=tasks["flags"],
            pg_id=pg_id, pg_valid=pg_valid, pg_pos=pg_pos, qt_list=qt_list,
            part_indptr=part_indptr, part_base=part_base, part_hstride=part_hstride,
            merge_qt=merge_qt,
        )

    # ---------------------------------------------------------------- tree-walk lists
    def walk_plan(self, leaves: Sequence[int], q_lens: Optional[Sequence[int]],
                  num_q_heads: int, num_kv_heads: int, row_tiles: int = 0,
                  waves: int = 0, draft_masks: Optional[Sequence[int]] = None) -> Dict[str, object]:
        L = len(leaves)
        q_lens = [1] * L if q_lens is None else list(q_lens)
        G = num_q_heads // num_kv_heads
        P = self.P
        paths = [self.path(u) for u in leaves]
        rows = [ql * G for ql in q_lens]
        none = dict(available=0, row_tiles=0, waves=0, row_blocks=[], blocks=[], qt=[], items=[])
        if L == 0:
            return none
        qoff, limits, first_unseen = [], [], []
        for path, ql in zip(paths, q_lens):
            T = sum(self.tokens[w] for w in path)
            qoff.append(len(limits))
            lead = 1
            if draft_masks is not None:
                mk = [int(x) for x in draft_masks[len(limits):len(limits) + ql]]
                lead = 0
                while lead < ql and all((x >> lead) & 1 for x in mk):
                    lead += 1
            first_unseen.append(T - ql + lead)
            limits += [T - ql + 1 + i for i in range(ql)]
        roots: List[int] = []
        for path in paths:
            if path[0] not in roots:
                roots.append(path[0])
        root_rows = {r: 0 for r in roots}
        for path, n in zip(paths, rows):
            root_rows[path[0]] += n
        if row_tiles == 0:
            if G > 64:
                return none
            if max(rows) <= 16:
                row_tiles = 1
                if max(root_rows.values()) > 64 and \
                        sum(-(-r // 128) for r in root_rows.values()) * num_kv_heads >= 512:
                    row_tiles = 2
            elif max(rows) <= 32:
                row_tiles = 2
            else:                      # wider requests are cut into pieces of whole query tokens
                row_tiles = 4 if G > 32 else 2
        elif G > 16 * row_tiles:
            return dict(none, row_tiles=0)
        if waves == 2 and row_tiles == 4:
            return none
        C = 16 * row_tiles
        NW = waves if waves else 4
        if waves == 0 and draft_masks is None and row_tiles <= 2 and max(rows) <= C \
                and max(root_rows.values()) > 4 * C \
                and sum(-(-r // (8 * C)) for r in root_rows.values()) * num_kv_heads >= 1024:
            NW = 8
        pos0: Dict[int, int] = {}
        for path in paths:
            t = 0
            for w in path:
                pos0[w] = t
                t += self.tokens[w]

        order = sorted(range(L), key=lambda i: (roots.index(paths[i][0]), paths[i], i))
        cap = C // G                   # query tokens a wavefront holds
        pieces: List[Tuple[int, int, int]] = []     # (request, first query token, tokens)
        for i in order:
            n_p = -(-q_lens[i] // cap)
            base, rem = divmod(q_lens[i], n_p)
            j0 = 0
            for k in range(n_p):
                n = base + (1 if k < rem else 0)
                pieces.append((i, j0, n))
                j0 += n
        qt: List[int] = []
        row_blocks: List[List[int]] = []
        blocks: List[List[int]] = []
        rb_total: List[int] = []
        rbs_of_root: Dict[int, List[int]] = {r: [] for r in roots}

        # row block of every request (same packing as below), then the nodes met by several
        rbs_through: Dict[int, set] = {}
        rb, cur_root, wave, used = -1, None, 0, 0
        for i, _, n in pieces:
            if paths[i][0] != cur_root:
                cur_root, rb, wave, used = paths[i][0], rb + 1, 0, 0
            elif used + n * G > C:
                wave, used = wave + 1, 0
                if wave == NW:
                    rb, wave = rb + 1, 0
            used += n * G
            for w in paths[i]:
                rbs_through.setdefault(w, set()).add(rb)

        def node_blocks(u, lo, hi, minlim):
            out = []
            multi = 2 if len(rbs_through[u]) > 1 else 0
            pages, valid = self.pages[u], self.node_page_valid(u)
            for k in range(0, len(pages), 2):
                has_b = k + 1 < len(pages)
                va, vb = valid[k], (valid[k + 1] if has_b else 0)
                pos_a = pos0[u] + k * P
                pos_b = pos_a + P
                end = pos_b + vb if has_b else pos_a + va
                masked = va != P or not has_b or vb != P or minlim < end
                out.append([pages[k], (pos_a << 7) | va, pages[k + 1] if has_b else pages[k],
                            ((pos_b << 7) | vb) if has_b else 0, lo | (hi << 16), int(masked) | multi, 0, 0])
            return out

        overflow: List[int] = []

        def flush(root, placed, qt_first, qt_count):
            if not placed:
                return
            nodes: Dict[int, List[int]] = {}          # insertion order = encounter order
            for i, row0, nrows in placed:
                for w in paths[i]:
                    if self.tokens[w] == 0:
                        continue
                    if w not in nodes:
                        nodes[w] = [row0, row0 + nrows, first_unseen[i]]
                    else:
                        nodes[w][1] = row0 + nrows
                        nodes[w][2] = min(nodes[w][2], first_unseen[i])
            first = len(blocks)
            shared = [b for w, (lo, hi, ml) in nodes.items() if lo // C != (hi - 1) // C
                      for b in node_blocks(w, lo, hi, ml)]
            blocks.extend(shared)
            n_priv, packed = [], []
            asked = {leaves[i] for i, _, _ in placed}
            for wv in range(NW):
                own = [w for w, (lo, hi, ml) in nodes.items() if lo // C == (hi - 1) // C and lo // C == wv]
                mine = [b for w in own for b in node_blocks(w, *nodes[w])]
                # room for blocks that appends will start: two records per requested childless node
                room = 2 * sum(1 for w in own if w in asked and not self.has_live_children(w))
                if len(mine) + room > 0xffff:
                    overflow.append(1)
                blocks.extend(mine)
                blocks.extend([[0] * 8 for _ in range(room)])
                n_priv.append(len(mine))
                packed.append(len(mine) | ((len(mine) + room) << 16))
            rbs_of_root[root].append(len(row_blocks))
            row_blocks.append([root, first, len(shared)] + packed + qt_first + qt_count)
            rb_total.append(len(shared) + sum(n_priv))

        cur_root, wave, used = None, 0, 0
        placed, qt_first, qt_count = [], [0] * NW, [0] * NW
        for i, j0, n in pieces:
            root = paths[i][0]
            if root != cur_root:
                flush(cur_root, placed, qt_first, qt_count)
                cur_root, wave, used = root, 0, 0
                placed, qt_first, qt_count = [], [0] * NW, [0] * NW
            elif used + n * G > C:
                wave, used = wave + 1, 0
                if wave == NW:
                    flush(cur_root, placed, qt_first, qt_count)
                    wave = 0
                    placed, qt_first, qt_count = [], [0] * NW, [0] * NW
            if qt_count[wave] == 0:
                qt_first[wave] = len(qt) // 2
            for j in range(j0, j0 + n):
                qt += [qoff[i] + j, limits[qoff[i] + j]]
            qt_count[wave] += n
            placed.append((i, wave * C + used, n * G))
            used += n * G
        flush(cur_root, placed, qt_first, qt_count)
        if overflow:
            return dict(available=0, row_tiles=0, waves=0, row_blocks=[], blocks=[], qt=[], items=[])

        root_blocks = {r: sum(rb_total[b] for b in rbs_of_root[r]) for r in roots}
        root_order = sorted(roots, key=lambda r: -root_blocks[r])      # stable
        lanes = 8 // num_kv_heads if num_kv_heads in (1, 2, 4) else 1
        lane_rbs: List[List[int]] = [[] for _ in range(lanes)]
        load = [0] * lanes
        for r in root_order:
            best = min(range(lanes), key=lambda l: (load[l], l))
            lane_rbs[best] += rbs_of_root[r]
            load[best] += root_blocks[r]
        items: List[int] = []
        for r in range(max(len(v) for v in lane_rbs)):
            for l in range(lanes):
                real = r < len(lane_rbs[l])
                if not real and lanes == 1:
                    continue
                for g in range(num_kv_heads):
                    stride = 16 if NW <= 4 else 32
                    if real:
                        rb = lane_rbs[l][r]
                        body = [g] + row_blocks[rb][1:]
                        items += body + [0] * (stride - 1 - len(body)) + [rb]
                    else:
                        items += [g] + [0] * (stride - 2) + [-1]
        return dict(available=1, row_tiles=row_tiles, waves=NW,
                    row_blocks=[x for rb in row_blocks for x in rb],
                    blocks=[x for b in blocks for x in b], qt=qt, items=items)
