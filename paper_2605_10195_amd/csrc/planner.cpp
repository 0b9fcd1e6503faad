#include "planner.hpp"

#include <algorithm>
#include <limits>
#include <numeric>
#include <unordered_set>
#include <utility>

namespace spex {
namespace {

constexpr int32_t kWaveRowsMax = 16;    // largest group the wavefront kernel takes
constexpr int kWideClass = 1;           // cooperative launch class of groups above 64 rows
constexpr int32_t kWideSpan = 64 << kWideClass;  // rows per workgroup in that class

int32_t clamp32(int64_t v, int32_t lo, int32_t hi) {
  return static_cast<int32_t>(std::max<int64_t>(lo, std::min<int64_t>(hi, v)));
}

struct Segment {
  std::vector<int32_t> ids, valid, pos;
  std::vector<int32_t> last_of;  // node whose last page the entry is, else -1
  int32_t qt_begin = 0, qt_count = 0;
};

}  // namespace

PlanError Planner::begin(const PageTable &pt, const int32_t *leaves, const int32_t *q_lens,
                         const uint32_t *draft_masks, int32_t n_leaves, int32_t num_q_heads,
                         int32_t num_kv_heads,
                         int32_t prefix_chunk_pages, int32_t suffix_chunk_pages,
                         int32_t walk_row_tiles, int32_t walk_waves, Plan *plan) {
  if (n_leaves < 0 || (n_leaves > 0 && !leaves)) return PlanError::kInvalid;
  const int32_t N = pt.num_nodes();
  Plan &pl = *plan;
  {
    // A fresh Plan, but the largest lists keep the memory of the previous plan: a request of
    // thousands of branches has megabytes of block records, and growing those vectors from
    // nothing each time costs more than filling them.
    std::vector<int32_t> *big[] = {&pl.walk_blocks, &pl.walk_items, &pl.walk_qt,   &pl.walk_rb,  &pl.path_nodes,
                                   &pl.path_indptr, &pl.qt_limit,   &pl.pg_rec,    &pl.qt_rec,   &pl.leaf_pages};
    constexpr int kBig = sizeof(big) / sizeof(big[0]);
    std::vector<int32_t> kept[kBig];
    for (int i = 0; i < kBig; ++i) {
      kept[i] = std::move(*big[i]);
      kept[i].clear();
    }
    pl = Plan();
    for (int i = 0; i < kBig; ++i) *big[i] = std::move(kept[i]);
  }
  pl.req_leaves.assign(leaves, leaves + n_leaves);
  if (q_lens) pl.req_q_lens.assign(q_lens, q_lens + n_leaves);
  pl.table_version = pt.version();
  pl.structure_version = pt.structure_version();
  pl.topology_version = pt.topology_version();
  pl.req_prefix_chunk = prefix_chunk_pages;
  pl.req_suffix_chunk = suffix_chunk_pages;
  pl.req_walk_row_tiles = walk_row_tiles;
  pl.req_walk_waves = walk_waves;
  pl.num_q_heads = num_q_heads;
  pl.num_kv_heads = num_kv_heads;

  if (static_cast<int32_t>(live_.size()) < N) {
    live_.resize(N, 0);
    pos0_.resize(N, 0);
    gindex_.resize(N, -1);
    last_pg_.resize(N, -1);
  }

  // ---- paths and limits
  if (static_cast<int32_t>(stamp_.size()) < N) {
    stamp_.resize(N, 0);
    slot_.resize(N, 0);
  }
  if (stamp_next_ == std::numeric_limits<int32_t>::max()) {
    std::fill(stamp_.begin(), stamp_.end(), 0);
    stamp_next_ = 1;
  }
  const int32_t st_seen = stamp_next_++;
  pl.path_indptr.assign(n_leaves + 1, 0);
  pl.qoff.assign(n_leaves, 0);
  pl.req_tokens.assign(n_leaves, 0);
  pl.req_minlim.assign(n_leaves, 0);
  std::vector<int32_t> tmp;
  for (int32_t i = 0; i < n_leaves; ++i) {
    const int32_t leaf = leaves[i];
    const int32_t ql = q_lens ? q_lens[i] : 1;
    if (!pt.valid(leaf)) return PlanError::kBadNode;
    tmp.clear();
    for (int32_t u = leaf; u != kNoNode; u = pt.node(u).parent) tmp.push_back(u);
    int64_t T = 0;
    for (auto it = tmp.rbegin(); it != tmp.rend(); ++it) {
      const int32_t u = *it;
      pl.path_nodes.push_back(u);
      pos0_[u] = static_cast<int32_t>(T);
      T += pt.node(u).n_tokens;
      if (stamp_[u] != st_seen) {
        stamp_[u] = st_seen;
        pl.unique_tokens += pt.node(u).n_tokens;
      }
    }
    pl.path_indptr[i + 1] = static_cast<int32_t>(pl.path_nodes.size());
    pl.req_tokens[i] = pt.node(leaf).n_tokens;
    if (ql < 1) return PlanError::kInvalid;
    if (ql > T) return PlanError::kEmptyPath;
    if (T >= (1 << 24)) return PlanError::kTooLarge;  // positions are packed in 24 bits
    pl.qoff[i] = static_cast<int32_t>(pl.qt_limit.size());
    for (int32_t j = 0; j < ql; ++j) pl.qt_limit.push_back(static_cast<int32_t>(T) - ql + 1 + j);
    int32_t lead = 1;
    if (draft_masks) {
      // Query j of the request sees every position before the q_len drafts and draft k iff bit k
      // of its mask is set.
      if (ql > 32) return PlanError::kInvalid;
      const uint32_t *mk = draft_masks + pl.qoff[i];
      uint32_t all = 0xffffffffu;
      for (int32_t j = 0; j < ql; ++j) {
        if (ql < 32 && (mk[j] >> ql) != 0) return PlanError::kInvalid;
        if (mk[j] == 0 && T == ql) return PlanError::kEmptyPath;
        all &= mk[j];
        pl.qt_mask.push_back(j);
        pl.qt_mask.push_back(static_cast<int32_t>(mk[j]));
      }
      lead = 0;
      while (lead < ql && ((all >> lead) & 1)) ++lead;
    }
    pl.req_minlim[i] = static_cast<int32_t>(T) - ql + lead;
  }
  if (draft_masks) pl.req_masks.assign(draft_masks, draft_masks + pl.qt_limit.size());
  pl.valid = true;
  return PlanError::kOk;
}

// Root-to-node page lists of the requested nodes (CSR); only the dump and the tests read them.
void Planner::ensure_csr(const PageTable &pt, Plan *plan) {
  Plan &pl = *plan;
  if (pl.has_csr) return;
  const int32_t n_leaves = static_cast<int32_t>(pl.req_leaves.size());
  pl.leaf_indptr.assign(1, 0);
  for (int32_t i = 0; i < n_leaves; ++i) {
    for (int32_t k = pl.path_indptr[i]; k < pl.path_indptr[i + 1]; ++k) {
      const int32_t u = pl.path_nodes[k];
      const Node &nd = pt.node(u);
      for (size_t pg = 0; pg < nd.pages.size(); ++pg) {
        pl.leaf_pages.push_back(nd.pages[pg]);
        pl.leaf_valid.push_back(pt.page_valid(u, static_cast<int32_t>(pg)));
      }
    }
    pl.leaf_indptr.push_back(static_cast<int32_t>(pl.leaf_pages.size()));
  }
  pl.has_csr = true;
}

// Shared-prefix groups, suffixes, chunks, partial slots, merge lists and the work items of the
// shared-prefix / suffix / merge kernels.
PlanError Planner::ensure_split(const PageTable &pt, Plan *plan) {
  Plan &pl = *plan;
  if (pl.has_split) return PlanError::kOk;
  const int32_t P = pt.page_size();
  const int32_t num_kv_heads = pl.num_kv_heads;
  const int32_t G = pl.num_q_heads / pl.num_kv_heads;
  const int32_t n_leaves = static_cast<int32_t>(pl.req_leaves.size());
  const int32_t *q_lens = pl.req_q_lens.empty() ? nullptr : pl.req_q_lens.data();
  const std::vector<int32_t> &path_indptr = pl.path_indptr, &path_nodes = pl.path_nodes, &qoff = pl.qoff;
  const int32_t prefix_chunk_pages = pl.req_prefix_chunk, suffix_chunk_pages = pl.req_suffix_chunk;
  auto reset = [&]() {
    for (int32_t u : touched_) {
      live_[u] = 0;
      gindex_[u] = -1;
      last_pg_[u] = -1;
    }
    touched_.clear();
  };
  for (int32_t k : path_nodes)
    if (live_[k]++ == 0) touched_.push_back(k);
  const int32_t NQ = static_cast<int32_t>(pl.qt_limit.size());

  // ---- groups
  for (int32_t u : touched_)
    if (live_[u] >= 2 && pt.node(u).n_tokens > 0) pl.group_node.push_back(u);
  std::sort(pl.group_node.begin(), pl.group_node.end());
  const int32_t NG = static_cast<int32_t>(pl.group_node.size());
  for (int32_t gi = 0; gi < NG; ++gi) gindex_[pl.group_node[gi]] = gi;
  std::vector<int32_t> group_count(NG, 0);
  for (int32_t i = 0; i < n_leaves; ++i) {
    const int32_t ql = q_lens ? q_lens[i] : 1;
    for (int32_t k = path_indptr[i]; k < path_indptr[i + 1]; ++k) {
      const int32_t gi = gindex_[path_nodes[k]];
      if (gi >= 0) group_count[gi] += ql;
    }
  }
  std::vector<int32_t> group_qt_begin(NG + 1, 0);
  for (int32_t gi = 0; gi < NG; ++gi) group_qt_begin[gi + 1] = group_qt_begin[gi] + group_count[gi];
  const int32_t n_group_qt = group_qt_begin[NG];
  pl.qt_list.assign(static_cast<size_t>(n_group_qt) + NQ, 0);
  std::vector<int32_t> fill(group_qt_begin.begin(), group_qt_begin.end() - 1);
  for (int32_t i = 0; i < n_leaves; ++i) {
    const int32_t ql = q_lens ? q_lens[i] : 1;
    for (int32_t k = path_indptr[i]; k < path_indptr[i + 1]; ++k) {
      const int32_t gi = gindex_[path_nodes[k]];
      if (gi < 0) continue;
      for (int32_t j = 0; j < ql; ++j) pl.qt_list[fill[gi]++] = qoff[i] + j;
    }
  }
  std::iota(pl.qt_list.begin() + n_group_qt, pl.qt_list.end(), 0);

  // ---- segments
  auto add_node_pages = [&](Segment &s, int32_t u) {
    const Node &nd = pt.node(u);
    int32_t t = pos0_[u];
    for (size_t k = 0; k < nd.pages.size(); ++k) {
      const int32_t v = pt.page_valid(u, static_cast<int32_t>(k));
      s.ids.push_back(nd.pages[k]);
      s.valid.push_back(v);
      s.pos.push_back(t);
      s.last_of.push_back(k + 1 == nd.pages.size() ? u : -1);
      t += v;
    }
  };
  std::vector<Segment> groups(NG), suffixes;
  int64_t prefix_pages_weighted = 0;
  int32_t max_rows_small = 0;
  for (int32_t gi = 0; gi < NG; ++gi) {
    add_node_pages(groups[gi], pl.group_node[gi]);
    groups[gi].qt_begin = group_qt_begin[gi];
    groups[gi].qt_count = group_count[gi];
    pl.max_rows_prefix = std::max(pl.max_rows_prefix, group_count[gi] * G);
    if (group_count[gi] * G <= kWaveRowsMax) max_rows_small = std::max(max_rows_small, group_count[gi] * G);
  }
  suffixes.reserve(n_leaves);
  int64_t suffix_pages = 0;
  for (int32_t i = 0; i < n_leaves; ++i) {
    const int32_t ql = q_lens ? q_lens[i] : 1;
    int32_t k0 = path_indptr[i + 1];
    while (k0 > path_indptr[i] && live_[path_nodes[k0 - 1]] == 1) --k0;
    Segment s;
    for (int32_t k = k0; k < path_indptr[i + 1]; ++k) add_node_pages(s, path_nodes[k]);
    if (s.ids.empty()) continue;
    s.qt_begin = n_group_qt + qoff[i];
    s.qt_count = ql;
    suffix_pages += static_cast<int64_t>(s.ids.size());
    pl.max_rows_suffix = std::max(pl.max_rows_suffix, ql * G);
    suffixes.push_back(std::move(s));
  }
  pl.prefix_row_tiles = max_rows_small <= 16 ? 1 : 2;
  pl.suffix_row_tiles = pl.max_rows_suffix <= 16 ? 1 : 2;
  const int32_t rw_suffix = 16 * pl.suffix_row_tiles;
  for (const Segment &s : groups)  // work items per page if nothing were split
    prefix_pages_weighted +=
        static_cast<int64_t>(s.ids.size()) * (s.qt_count * G <= 64 ? 1 : (s.qt_count * G + kWideSpan - 1) / kWideSpan);

  // ---- split granularity.  Every extra chunk costs a partial result per row that is written and
  // read back, so segments are cut only as far as needed to keep the longest work item near
  // 1/1024 (shared prefix) or 1/2048 (suffix) of the launch, i.e. a few items per wavefront slot.
  pl.prefix_chunk_pages = prefix_chunk_pages > 0
                              ? prefix_chunk_pages
                              : clamp32((prefix_pages_weighted * num_kv_heads + 1023) / 1024, 16, 256);
  pl.suffix_chunk_pages = suffix_chunk_pages > 0
                              ? suffix_chunk_pages
                              : clamp32((suffix_pages * num_kv_heads + 2047) / 2048, 8, 64);

  // ---- tasks
  std::vector<int32_t> qt_req;  // with draft masks: the request of every query token
  if (!pl.qt_mask.empty()) {
    qt_req.resize(NQ);
    for (int32_t i = 0; i < n_leaves; ++i)
      for (int32_t j = 0; j < (q_lens ? q_lens[i] : 1); ++j) qt_req[qoff[i] + j] = i;
  }
  std::vector<std::vector<std::pair<int32_t, int32_t>>> parts(NQ);
  int64_t pbase = 0;
  bool overflow = false;
  auto emit = [&](const Segment &s, int32_t chunk_pages, int64_t *tokens, bool suffix) -> bool {
    const int32_t n = static_cast<int32_t>(s.ids.size());
    const int32_t rows = s.qt_count * G;
    // first path position that some row of the task does not see: the smallest limit for the
    // causal chain; with draft masks a query may miss drafts below its own position, and the
    // request's first position not seen by all its queries takes the limit's place
    int32_t min_limit = std::numeric_limits<int32_t>::max();
    for (int32_t r = 0; r < s.qt_count; ++r) {
      const int32_t qt = pl.qt_list[s.qt_begin + r];
      min_limit = std::min(min_limit, qt_req.empty() ? pl.qt_limit[qt] : pl.req_minlim[qt_req[qt]]);
    }
    const int32_t c = (n + chunk_pages - 1) / chunk_pages;
    const bool final = suffix && c == 1;
    for (int32_t j = 0; j < c; ++j) {
      const int32_t a = static_cast<int32_t>(static_cast<int64_t>(j) * n / c);
      const int32_t b = static_cast<int32_t>(static_cast<int64_t>(j + 1) * n / c);
      bool masked = min_limit < s.pos[b - 1] + s.valid[b - 1];
      for (int32_t k = a; k < b; ++k) {
        masked = masked || s.valid[k] != P;
        *tokens += s.valid[k];
      }
      if (pbase > std::numeric_limits<int32_t>::max() - static_cast<int64_t>(rows) * num_kv_heads)
        overflow = true;
      pl.task_pg_begin.push_back(static_cast<int32_t>(pl.pg_id.size()));
      pl.task_pg_count.push_back(b - a);
      pl.task_qt_begin.push_back(s.qt_begin);
      pl.task_qt_count.push_back(s.qt_count);
      pl.task_pbase.push_back(static_cast<int32_t>(pbase));
      pl.task_flags.push_back((masked ? 1 : 0) | (final ? 2 : 0));
      pl.pg_id.insert(pl.pg_id.end(), s.ids.begin() + a, s.ids.begin() + b);
      pl.pg_valid.insert(pl.pg_valid.end(), s.valid.begin() + a, s.valid.begin() + b);
      pl.pg_pos.insert(pl.pg_pos.end(), s.pos.begin() + a, s.pos.begin() + b);
      for (int32_t k = a; k < b; ++k)
        if (s.last_of[k] >= 0) last_pg_[s.last_of[k]] = static_cast<int32_t>(pl.pg_id.size()) - (b - k);
      for (int32_t r = 0; r < s.qt_count; ++r)
        parts[pl.qt_list[s.qt_begin + r]].emplace_back(static_cast<int32_t>(pbase) + r * G, rows);
      pbase += static_cast<int64_t>(rows) * num_kv_heads;
    }
    return final;
  };
  for (const Segment &s : groups) emit(s, pl.prefix_chunk_pages, &pl.prefix_tokens, false);
  pl.n_prefix_tasks = static_cast<int32_t>(pl.task_pbase.size());
  {
    std::vector<char> is_final(NQ, 0);
    for (const Segment &s : suffixes)
      if (emit(s, pl.suffix_chunk_pages, &pl.suffix_tokens, true))
        for (int32_t r = 0; r < s.qt_count; ++r) is_final[pl.qt_list[s.qt_begin + r]] = 1;
    for (int32_t t = 0; t < NQ; ++t)
      if (!is_final[t]) pl.merge_qt.push_back(t);
  }
  pl.n_partial_rows = pbase;
  // Where an append to a requested node shows up: the page entry of its last page, whether that
  // entry belongs to a group, and the positions of its query tokens in qt_list.
  pl.req_split_pg.assign(n_leaves, -1);
  pl.req_in_group.assign(n_leaves, 0);
  pl.req_qtpos_indptr.assign(1, 0);
  {
    std::vector<int32_t> fill2(group_qt_begin.begin(), group_qt_begin.end() - 1);
    for (int32_t i = 0; i < n_leaves; ++i) {
      const int32_t ql = q_lens ? q_lens[i] : 1;
      const int32_t u = pl.req_leaves[i];
      pl.req_split_pg[i] = last_pg_[u];
      pl.req_in_group[i] = gindex_[u] >= 0 ? 1 : 0;
      for (int32_t k = path_indptr[i]; k < path_indptr[i + 1]; ++k) {
        const int32_t gi = gindex_[path_nodes[k]];
        if (gi < 0) continue;
        pl.req_qtpos.push_back(fill2[gi]);
        fill2[gi] += ql;
      }
      pl.req_qtpos.push_back(n_group_qt + qoff[i]);
      pl.req_qtpos_indptr.push_back(static_cast<int32_t>(pl.req_qtpos.size()));
    }
  }
  reset();
  if (overflow) {
    pl.valid = false;
    return PlanError::kTooLarge;
  }

  pl.part_indptr.assign(1, 0);
  for (const auto &lst : parts) {
    for (const auto &e : lst) {
      pl.part_base.push_back(e.first);
      pl.part_hstride.push_back(e.second);
    }
    pl.part_indptr.push_back(static_cast<int32_t>(pl.part_base.size()));
  }

  // ---- launch lists, heaviest tasks first
  const int32_t n_tasks = static_cast<int32_t>(pl.task_pbase.size());
  auto order_of = [&](int32_t lo, int32_t hi) {
    std::vector<int32_t> ord(hi - lo);
    std::iota(ord.begin(), ord.end(), lo);
    std::stable_sort(ord.begin(), ord.end(), [&](int32_t x, int32_t y) {
      return static_cast<int64_t>(pl.task_pg_count[x]) * pl.task_qt_count[x] >
             static_cast<int64_t>(pl.task_pg_count[y]) * pl.task_qt_count[y];
    });
    return ord;
  };
  auto push_item = [&](std::vector<int32_t> &items, int32_t t, int32_t g, int32_t row0) {
    const int32_t rec[Plan::kItemInts] = {pl.task_pg_begin[t], pl.task_pg_count[t],
                                          pl.task_qt_begin[t], pl.task_qt_count[t],
                                          pl.task_pbase[t],    pl.task_flags[t], g, row0};
    items.insert(items.end(), rec, rec + Plan::kItemInts);
  };
  // Shared-prefix items.  Groups of up to 16 rows go to the wavefront kernel (one item per task
  // and kv head).  Larger groups go to the cooperative kernel, one workgroup per (task, kv head,
  // span of 64 * NTW rows): NTW = 1 for up to 64 rows, else NTW = 2 (spans of 128 rows).
  // The spans of one (task, kv head) read the same pages; workgroup b of a launch runs on XCD
  // b % 8 and every XCD has its own L2, so units are laid out in batches of 8 with span s of unit
  // u at position s * 8 + u of the batch: all spans of a unit land on one XCD, next to each other
  // in dispatch order.  Holes are padding items (pg_count = 0).
  {
    constexpr int kXcds = 8;
    const int32_t empty_rec[Plan::kItemInts] = {0, 0, 0, 0, 0, 0, 0, 0};
    struct Unit { int32_t t, g, spans; };
    std::vector<Unit> wide;
    for (int32_t t : order_of(0, pl.n_prefix_tasks)) {
      const int32_t rows = pl.task_qt_count[t] * G;
      for (int32_t g = 0; g < num_kv_heads; ++g) {
        if (rows <= kWaveRowsMax) push_item(pl.prefix_items, t, g, 0);
        else if (rows <= 64) push_item(pl.coop_items[0], t, g, 0);
        else wide.push_back({t, g, (rows + kWideSpan - 1) / kWideSpan});
      }
    }
    for (size_t u0 = 0; u0 < wide.size(); u0 += kXcds) {
      const size_t n = std::min<size_t>(kXcds, wide.size() - u0);
      int32_t max_spans = 0;
      for (size_t k = 0; k < n; ++k) max_spans = std::max(max_spans, wide[u0 + k].spans);
      for (int32_t sidx = 0; sidx < max_spans; ++sidx)
        for (size_t k = 0; k < kXcds; ++k) {
          if (k < n && sidx < wide[u0 + k].spans)
            push_item(pl.coop_items[kWideClass], wide[u0 + k].t, wide[u0 + k].g, sidx * kWideSpan);
          else if (max_spans > 1)  // keep the XCD alignment inside the batch
            pl.coop_items[kWideClass].insert(pl.coop_items[kWideClass].end(), empty_rec,
                                             empty_rec + Plan::kItemInts);
        }
    }
  }
  for (int32_t t : order_of(pl.n_prefix_tasks, n_tasks)) {
    const int32_t n_rt = (pl.task_qt_count[t] * G + rw_suffix - 1) / rw_suffix;
    for (int32_t rt = 0; rt < n_rt; ++rt)
      for (int32_t g = 0; g < num_kv_heads; ++g) push_item(pl.suffix_items, t, g, rt * rw_suffix);
  }
  pl.pg_rec.resize(pl.pg_id.size() * 2);
  for (size_t i = 0; i < pl.pg_id.size(); ++i) {
    pl.pg_rec[2 * i] = pl.pg_id[i];
    pl.pg_rec[2 * i + 1] = (pl.pg_pos[i] << 7) | pl.pg_valid[i];
  }
  pl.qt_rec.resize(pl.qt_list.size() * 2);
  for (size_t i = 0; i < pl.qt_list.size(); ++i) {
    pl.qt_rec[2 * i] = pl.qt_list[i];
    pl.qt_rec[2 * i + 1] = pl.qt_limit[pl.qt_list[i]];
  }
  pl.has_split = true;
  return PlanError::kOk;
}

// Tree-walk lists: the whole path of a set of query rows is handled by one workgroup, which keeps
// the rows' softmax state in registers from the root to the requested nodes, so nothing is
// written but the output.  Rules (they fix the result uniquely):
//  * request i has q_len_i * G rows; C = 16 * NTW rows fit one wavefront.  NTW is the value asked
//    for (1, 2 or 4) or, if 0: 1 if no request has more than 16 rows (raised to 2 when some root
//    has more than 64 rows below it and sum over roots of ceil(rows / 128), times Hkv, is at least
//    512), 2 if none has more than 32, else 2 (4 if G > 32).  No lists (walk_ok = false) if
//    G > 16 * NTW, i.e. if one query token does not fit a wavefront, or if NW = 2 is asked for and NTW is 4.
//  * roots in order of first appearance in the request list; the requests of a root sorted by
//    path (node ids root first, lexicographic, a proper prefix first), ties in request order;
//    so the requests below any node are consecutive.
//  * a request with more than cap = C / G query tokens is cut into ceil(q_len / cap) pieces of
//    consecutive query tokens, the first (q_len mod pieces) of them one token longer than the
//    others; "request" in the rules below means such a piece.
//  * a row block has NW wavefronts of rows: the value asked for (2, 4 or 8); if 0: 8 if there are no
//    draft masks, NTW <= 2, no request has more than C rows, some root has more than 4 C rows and
//    sum over roots of ceil(rows / (8 C)), times Hkv, is at least 1024; else 4.  (With 2 the
//    kernel still runs four wavefronts: two per wavefront of rows, which split the path between them.)
//  * packing: a request joins the current wavefront if its rows still fit, else it starts the
//    next one; wavefront NW, or a new root, starts a new row block.  walk_qt lists
//    {query token, limit} of the requests in this order.  Wavefronts without requests have
//    first entry 0 and count 0.  Row of a request in its row block: wavefront * C + rows before
//    it in the wavefront.
//  * nodes of a row block: the nodes with >= 1 token on its requests' paths, in order of first
//    encounter (requests in order, each path root first), each with the row range
//    [first row of the first request through it, last row + 1 of the last request through it)
//    and minlim = min over those requests of the first path position some query of the request
//    does not see (T - q_len + 1 for the causal chain).  A node whose range touches two
//    wavefronts is shared, else it is private to wavefront lo / C.
//  * blocks of a row block: its shared nodes in encounter order, then the private nodes of
//    wavefront 0, 1, .., each wavefront's blocks followed by room for blocks that appends will
//    start: two all-zero records for every private node of the wavefront that a request of the
//    row block asks for and that has no live children; the row block and the work items hold
//    count | (count + room) << 16 per wavefront.  A node's pages two at a time (the last block
//    of an odd run has no page b).  Flag bit 0: page a or b partial, or no page b, or minlim smaller than the path
//    position after the block's last token.  Flag bit 1: the node lies on paths of more than one
//    row block (its pages are fetched again by another workgroup and are worth keeping cached).
//  * launch order: roots by descending number of blocks in their row blocks (stable).  With
//    lanes = 8 / Hkv for Hkv in {1, 2, 4}, else 1, every root in that order goes to the lane with the
//    fewest blocks so far (lowest index on ties) and appends its row blocks to it; round r emits,
//    for lane 0, 1, ..: the lane's r-th row block, or padding if the lane has run out and more
//    than one lane exists; each for kv head 0 .. Hkv-1.  Workgroup b runs on XCD b % 8, so the row
//    blocks of one root and kv head follow each other on one XCD and share its L2.
void Planner::ensure_walk(const PageTable &pt, Plan *plan) {
  if (plan->has_walk) return;
  plan->has_walk = true;
  const int32_t n_leaves = static_cast<int32_t>(plan->req_leaves.size());
  const int32_t *q_lens = plan->req_q_lens.empty() ? nullptr : plan->req_q_lens.data();
  const int32_t num_kv_heads = plan->num_kv_heads, G = plan->num_q_heads / plan->num_kv_heads;
  const int32_t walk_row_tiles = plan->req_walk_row_tiles, walk_waves = plan->req_walk_waves;
  const std::vector<int32_t> &path_indptr = plan->path_indptr, &path_nodes = plan->path_nodes,
                             &qoff = plan->qoff;
  Plan &pl = *plan;
  pl.walk_ok = false;
  pl.walk_row_tiles = 0;
  pl.walk_waves = 0;
  if (n_leaves == 0) return;
  const int32_t P = pt.page_size();
  const int32_t N = pt.num_nodes();
  if (static_cast<int32_t>(stamp_.size()) < N) {
    stamp_.resize(N, 0);
    slot_.resize(N, 0);
  }
  auto fresh = [&]() {
    if (stamp_next_ == std::numeric_limits<int32_t>::max()) {
      std::fill(stamp_.begin(), stamp_.end(), 0);
      stamp_next_ = 1;
    }
    return stamp_next_++;
  };
  auto rows_of = [&](int32_t i) { return (q_lens ? q_lens[i] : 1) * G; };

  int32_t max_rows = 0;
  std::vector<int32_t> root_of(n_leaves), root_ids;
  std::vector<int64_t> root_rows;
  {
    const int32_t st = fresh();
    for (int32_t i = 0; i < n_leaves; ++i) {
      max_rows = std::max(max_rows, rows_of(i));
      const int32_t r = path_nodes[path_indptr[i]];
      if (stamp_[r] != st) {
        stamp_[r] = st;
        slot_[r] = static_cast<int32_t>(root_ids.size());
        root_ids.push_back(r);
        root_rows.push_back(0);
      }
      root_of[i] = slot_[r];
      root_rows[slot_[r]] += rows_of(i);
    }
  }
  int32_t ntw = walk_row_tiles;
  if (ntw == 0) {
    if (G > 64) return;
    if (max_rows <= 16) {
      ntw = 1;
      if (*std::max_element(root_rows.begin(), root_rows.end()) > 64) {
        // Two tiles per wavefront halve the number of row blocks that walk a wide root's shared
        // pages -- worth it only if the launch still has at least two workgroups per compute unit
        // (512); below that, more and shorter workgroups balance better.
        int64_t wide_items = 0;
        for (int64_t r : root_rows) wide_items += (r + 127) / 128;
        if (wide_items * num_kv_heads >= 512) ntw = 2;
      }
    } else if (max_rows <= 32) {
      ntw = 2;
    } else {
      // Wider requests are cut into pieces (below).  Four tiles per wavefront leave one wavefront
      // per SIMD and were the slowest choice measured, so they are taken only when one query
      // token alone needs them.
      ntw = G > 32 ? 4 : 2;
    }
  } else if (G > 16 * ntw) {
    return;
  }
  if (walk_waves == 2 && ntw == 4) return;  // the kernel that splits the path holds at most two row tiles
  pl.walk_row_tiles = ntw;
  pl.req_walk_qt.assign(n_leaves, -1);
  pl.req_walk_home.assign(n_leaves, -2);
  pl.req_pages.resize(n_leaves);
  for (int32_t i = 0; i < n_leaves; ++i)
    pl.req_pages[i] = static_cast<int32_t>(pt.node(pl.req_leaves[i]).pages.size());
  bool room_overflow = false;
  const int32_t C = 16 * ntw;
  // Measured on MI355X, two workgroups of 4 wavefronts per compute unit beat one of 8 wherever a
  // root's rows fit one 4-wavefront row block (the barrier of the shared phase then stalls only
  // half of the unit), so 4 is the default.
  int32_t NW = walk_waves == 0 ? 4 : walk_waves;
  if (walk_waves == 0 && plan->req_masks.empty() && ntw <= 2 && max_rows <= C) {
    // Eight wavefronts: a root whose rows overflow one row block of four wavefronts gets row blocks
    // twice as large, so its shared pages are fetched by half as many workgroups (256 queries of
    // 32 branches and 8 rows each: once instead of twice, 1.04 instead of 1.16 times the unique
    // bytes), and since workgroups alternate in which kind of block they take first, the two
    // halves of such a root need not be in the same phase at the same time to share its prompt
    // in L2 (1.91 against 2.09 ms).  Only when no request is cut into pieces and at least 1024
    // such workgroups remain.
    bool wide = false;
    int64_t n8 = 0;
    for (int64_t r : root_rows) {
      wide = wide || r > 4 * C;
      n8 += (r + 8 * C - 1) / (8 * C);
    }
    if (wide && n8 * num_kv_heads >= 1024) NW = 8;
  }
  pl.walk_waves = NW;
  const int32_t rb_ints = 3 + 3 * NW, item_ints = NW <= 4 ? 16 : 32;

  // Order of the requests: by root, then by path (node ids root first, lexicographic, a proper
  // prefix first), ties in request order.  Comparing paths pairwise costs a walk over the common
  // prefix per comparison; instead every node on a requested path gets its rank in the pre-order
  // traversal of the requested part of the forest that visits roots in order of first appearance
  // and children in ascending id -- the same order -- and the requests are sorted by the rank of
  // their node.
  std::vector<int32_t> order(n_leaves);
  {
    if (static_cast<int32_t>(rank_.size()) < N) {
      rank_.resize(N, 0);
      child_lo_.resize(N, 0);
      child_n_.resize(N, 0);
    }
    const int32_t st_seen = fresh();
    edges_.clear();
    for (int32_t i = 0; i < n_leaves; ++i)
      for (int32_t k = path_indptr[i + 1] - 1; k >= path_indptr[i]; --k) {
        const int32_t u = path_nodes[k];
        if (stamp_[u] == st_seen) break;  // the rest of the path is known already
        stamp_[u] = st_seen;
        child_n_[u] = 0;
        if (k > path_indptr[i]) edges_.emplace_back(path_nodes[k - 1], u);
      }
    std::sort(edges_.begin(), edges_.end());
    for (size_t e = 0; e < edges_.size(); ++e) {
      const int32_t par = edges_[e].first;
      if (child_n_[par]++ == 0) child_lo_[par] = static_cast<int32_t>(e);
    }
    int32_t next_rank = 0;
    dfs_.clear();
    for (int32_t r = static_cast<int32_t>(root_ids.size()) - 1; r >= 0; --r) dfs_.push_back(root_ids[r]);
    while (!dfs_.empty()) {
      const int32_t u = dfs_.back();
      dfs_.pop_back();
      rank_[u] = next_rank++;
      for (int32_t c = child_n_[u] - 1; c >= 0; --c) dfs_.push_back(edges_[child_lo_[u] + c].second);
    }
    keyed_.resize(n_leaves);
    for (int32_t i = 0; i < n_leaves; ++i)
      keyed_[i] = (static_cast<int64_t>(rank_[path_nodes[path_indptr[i + 1] - 1]]) << 32) | static_cast<uint32_t>(i);
    std::sort(keyed_.begin(), keyed_.end());
    for (int32_t i = 0; i < n_leaves; ++i) order[i] = static_cast<int32_t>(keyed_[i] & 0xffffffff);
  }

  // A request with more query tokens than a wavefront holds is cut into pieces of consecutive
  // query tokens of (almost) equal size; the packing below places pieces.
  struct Piece { int32_t req, j0, n; };
  std::vector<Piece> pieces;
  pieces.reserve(n_leaves);
  {
    const int32_t cap = C / G;
    for (int32_t idx : order) {
      const int32_t ql = q_lens ? q_lens[idx] : 1;
      const int32_t n_p = (ql + cap - 1) / cap, base = ql / n_p, rem = ql % n_p;
      for (int32_t k = 0, j0 = 0; k < n_p; ++k) {
        const int32_t n = base + (k < rem ? 1 : 0);
        pieces.push_back({idx, j0, n});
        j0 += n;
      }
    }
  }

  // Nodes that lie on paths of more than one row block (same packing as below, counted first).
  if (static_cast<int32_t>(multi_.size()) < N) multi_.resize(N, 0);
  const int32_t st_multi = fresh();
  {
    const int32_t st_seen = fresh();
    int32_t wave = 0, used = 0, cur_root = -1, rb = -1;
    for (const Piece &pc : pieces) {
      const int32_t idx = pc.req, rows = pc.n * G;
      if (root_of[idx] != cur_root) {
        cur_root = root_of[idx];
        ++rb;
        wave = used = 0;
      } else if (used + rows > C) {
        ++wave;
        used = 0;
        if (wave == NW) {
          ++rb;
          wave = 0;
        }
      }
      used += rows;
      for (int32_t k = path_indptr[idx]; k < path_indptr[idx + 1]; ++k) {
        const int32_t u = path_nodes[k];
        if (stamp_[u] != st_seen) {
          stamp_[u] = st_seen;
          slot_[u] = rb;
        } else if (slot_[u] != rb) {
          multi_[u] = st_multi;
        }
      }
    }
  }

  const int32_t c_shift = ntw == 1 ? 4 : (ntw == 2 ? 5 : 6);  // C = 16 * ntw = 1 << c_shift
  struct Placed { int32_t req, row0, rows; };
  std::vector<std::pair<int32_t, int32_t>> last_blks;  // (request, block with its node's last page)
  struct NodeRange { int32_t node, lo, hi, minlim; };
  std::vector<Placed> cur;
  std::vector<NodeRange> nodes;
  std::vector<int64_t> rb_blocks;           // blocks per row block
  std::vector<std::vector<int32_t>> rbs_of_root(root_ids.size());
  std::vector<int32_t> rb_rec(rb_ints);
  auto start_rb = [&](int32_t root_slot) {
    for (int32_t &x : rb_rec) x = 0;
    rb_rec[0] = root_ids[root_slot];
    cur.clear();
  };
  int32_t last_blk_of_node = -1;  // set by emit_node: block that holds the node's last page
  auto emit_node = [&](const NodeRange &nr) -> int32_t {
    const Node &nd = pt.node(nr.node);
    last_blk_of_node = -1;
    const int32_t n = static_cast<int32_t>(nd.pages.size());
    const int32_t made = (n + 1) >> 1;
    if (made == 0) return 0;
    const size_t first = pl.walk_blocks.size();
    pl.walk_blocks.resize(first + static_cast<size_t>(made) * Plan::kBlockInts);
    int32_t *rec = &pl.walk_blocks[first];
    const int32_t *pages = nd.pages.data();
    const int32_t rows = nr.lo | (nr.hi << 16), multi = multi_[nr.node] == st_multi ? 2 : 0;
    const int32_t last_valid = nd.n_tokens - (n - 1) * P;  // every page but the last is full
    int32_t pos_a = pos0_[nr.node];
    for (int32_t k = 0; k < n; k += 2, rec += Plan::kBlockInts, pos_a += 2 * P) {
      const bool has_b = k + 1 < n;
      const int32_t va = k == n - 1 ? last_valid : P;
      const int32_t vb = has_b ? (k + 1 == n - 1 ? last_valid : P) : 0;
      const int32_t pos_b = pos_a + P;
      const int32_t end = has_b ? pos_b + vb : pos_a + va;
      const bool masked = va != P || !has_b || vb != P || nr.minlim < end;
      rec[0] = pages[k];
      rec[1] = (pos_a << 7) | va;
      rec[2] = has_b ? pages[k + 1] : pages[k];
      rec[3] = has_b ? ((pos_b << 7) | vb) : 0;
      rec[4] = rows;
      rec[5] = (masked ? 1 : 0) | multi;
      rec[6] = 0;
      rec[7] = 0;
    }
    last_blk_of_node = static_cast<int32_t>(first / Plan::kBlockInts) + made - 1;
    return made;
  };
  auto flush = [&](int32_t root_slot) {
    if (cur.empty()) return;
    const int32_t st = fresh();
    nodes.clear();
    for (const Placed &pc : cur) {
      const int32_t i = pc.req, rows = pc.rows, minlim = pl.req_minlim[i];
      for (int32_t k = path_indptr[i]; k < path_indptr[i + 1]; ++k) {
        const int32_t u = path_nodes[k];
        if (pt.node(u).n_tokens == 0) continue;
        if (stamp_[u] != st) {
          stamp_[u] = st;
          slot_[u] = static_cast<int32_t>(nodes.size());
          nodes.push_back({u, pc.row0, pc.row0 + rows, minlim});
        } else {
          NodeRange &nr = nodes[slot_[u]];
          nr.hi = pc.row0 + rows;
          nr.minlim = std::min(nr.minlim, minlim);
        }
      }
    }
    rb_rec[1] = static_cast<int32_t>(pl.walk_blocks.size() / Plan::kBlockInts);
    int64_t total = 0;
    const int32_t rb_index = static_cast<int32_t>(pl.walk_rb.size() / rb_ints);
    // requests of this row block that asked for nr.node; home: the wavefront whose private list
    // holds the node (-1: a shared node).  Returns whether any request asked for it.
    // The placed requests that ask for one node follow each other (the requests are in path
    // order): first index and count per asked node, in the per-node scratch of the ordering step.
    for (int32_t ci = 0; ci < static_cast<int32_t>(cur.size()); ++ci) {
      const int32_t u = pl.req_leaves[cur[ci].req];
      if (rank_[u] != -st) {
        rank_[u] = -st;  // ranks are >= 0 and no longer needed: a negative stamp marks "asked in this row block"
        child_lo_[u] = ci;
        child_n_[u] = 0;
      }
      ++child_n_[u];
    }
    auto note_last = [&](const NodeRange &nr, int32_t home) {
      if (rank_[nr.node] != -st) return false;
      for (int32_t ci = child_lo_[nr.node]; ci < child_lo_[nr.node] + child_n_[nr.node]; ++ci) {
        const Placed &pc = cur[ci];
        if (last_blks.empty() || last_blks.back() != std::make_pair(pc.req, last_blk_of_node)) {
          last_blks.emplace_back(pc.req, last_blk_of_node);
          int32_t &h = pl.req_walk_home[pc.req];
          h = (h == -2 && home >= 0) ? rb_index * NW + home : -1;
        }
      }
      return true;
    };
    // wavefront that holds all rows of a node, or -1 if they touch several (C is a power of two)
    auto home_of = [&](const NodeRange &nr) { return (nr.lo >> c_shift) == ((nr.hi - 1) >> c_shift) ? (nr.lo >> c_shift) : -1; };
    for (const NodeRange &nr : nodes)
      if (home_of(nr) < 0) {
        rb_rec[2] += emit_node(nr);
        note_last(nr, -1);
      }
    total += rb_rec[2];
    int32_t longest_private = 0;
    for (int32_t w = 0; w < NW; ++w) {
      int32_t count = 0, room = 0;
      for (const NodeRange &nr : nodes)
        if (home_of(nr) == w) {
          count += emit_node(nr);
          if (note_last(nr, w) && pt.node(nr.node).n_live_children == 0) room += 2;
        }
      pl.walk_blocks.resize(pl.walk_blocks.size() + static_cast<size_t>(room) * Plan::kBlockInts, 0);
      if (count + room > 0xffff) room_overflow = true;
      rb_rec[3 + w] = count | ((count + room) << 16);
      total += count;
      longest_private = std::max(longest_private, count);
    }
    rbs_of_root[root_slot].push_back(static_cast<int32_t>(pl.walk_rb.size() / rb_ints));
    pl.walk_rb.insert(pl.walk_rb.end(), rb_rec.begin(), rb_rec.end());
    rb_blocks.push_back(total);
    pl.walk_block_visits += total;
    pl.walk_max_item_blocks = std::max(pl.walk_max_item_blocks, rb_rec[2] + longest_private);
  };

  int32_t wave = 0, used = 0, cur_root = -1;
  for (const Piece &piece : pieces) {
    const int32_t idx = piece.req, rows = piece.n * G;
    if (root_of[idx] != cur_root) {
      if (cur_root >= 0) flush(cur_root);
      cur_root = root_of[idx];
      start_rb(cur_root);
      wave = used = 0;
    } else if (used + rows > C) {
      ++wave;
      used = 0;
      if (wave == NW) {
        flush(cur_root);
        start_rb(cur_root);
        wave = 0;
      }
    }
    if (rb_rec[3 + 2 * NW + wave] == 0) rb_rec[3 + NW + wave] = static_cast<int32_t>(pl.walk_qt.size() / 2);
    // the pieces of a request follow each other, so its entries in walk_qt are consecutive
    if (piece.j0 == 0) pl.req_walk_qt[idx] = static_cast<int32_t>(pl.walk_qt.size() / 2);
    for (int32_t j = piece.j0; j < piece.j0 + piece.n; ++j) {
      pl.walk_qt.push_back(qoff[idx] + j);
      pl.walk_qt.push_back(pl.qt_limit[qoff[idx] + j]);
    }
    rb_rec[3 + 2 * NW + wave] += piece.n;
    cur.push_back({idx, wave * C + used, rows});
    used += rows;
  }
  flush(cur_root);
  // blocks to patch when a requested node grows: one per row block that holds a piece of the request
  pl.req_walk_blk_indptr.assign(n_leaves + 1, 0);
  for (const auto &rb : last_blks) ++pl.req_walk_blk_indptr[rb.first + 1];
  for (int32_t i = 0; i < n_leaves; ++i) pl.req_walk_blk_indptr[i + 1] += pl.req_walk_blk_indptr[i];
  pl.req_walk_blk.assign(last_blks.size(), -1);
  {
    std::vector<int32_t> fill(pl.req_walk_blk_indptr.begin(), pl.req_walk_blk_indptr.end() - 1);
    for (const auto &rb : last_blks) pl.req_walk_blk[fill[rb.first]++] = rb.second;
  }

  for (int32_t &h : pl.req_walk_home)
    if (h == -2) h = -1;
  if (room_overflow) return;  // a wavefront with more than 65535 private blocks: no tree-walk lists

  // ---- launch order
  const int32_t n_roots = static_cast<int32_t>(root_ids.size());
  std::vector<int64_t> root_blocks(n_roots, 0);
  for (int32_t r = 0; r < n_roots; ++r)
    for (int32_t rb : rbs_of_root[r]) root_blocks[r] += rb_blocks[rb];
  std::vector<int32_t> root_order(n_roots);
  std::iota(root_order.begin(), root_order.end(), 0);
  std::stable_sort(root_order.begin(), root_order.end(),
                   [&](int32_t a, int32_t b) { return root_blocks[a] > root_blocks[b]; });
  const int32_t lanes = (num_kv_heads == 1 || num_kv_heads == 2 || num_kv_heads == 4) ? 8 / num_kv_heads : 1;
  std::vector<std::vector<int32_t>> lane_rbs(lanes);
  std::vector<int64_t> lane_load(lanes, 0);
  for (int32_t r : root_order) {
    int32_t best = 0;
    for (int32_t l = 1; l < lanes; ++l)
      if (lane_load[l] < lane_load[best]) best = l;
    lane_rbs[best].insert(lane_rbs[best].end(), rbs_of_root[r].begin(), rbs_of_root[r].end());
    lane_load[best] += root_blocks[r];
  }
  size_t rounds = 0;
  for (const auto &v : lane_rbs) rounds = std::max(rounds, v.size());
  pl.rb_item0.assign(pl.walk_rb.size() / rb_ints, -1);
  for (size_t r = 0; r < rounds; ++r)
    for (int32_t l = 0; l < lanes; ++l) {
      const bool real = r < lane_rbs[l].size();
      if (!real && lanes == 1) continue;
      for (int32_t g = 0; g < num_kv_heads; ++g) {
        const size_t at = pl.walk_items.size();
        pl.walk_items.resize(at + item_ints, 0);
        int32_t *rec = &pl.walk_items[at];
        rec[0] = g;
        rec[item_ints - 1] = -1;
        if (real) {
          const int32_t rb = lane_rbs[l][r];
          for (int k = 1; k < rb_ints; ++k) rec[k] = pl.walk_rb[static_cast<size_t>(rb) * rb_ints + k];
          rec[item_ints - 1] = rb;
          if (g == 0) pl.rb_item0[rb] = static_cast<int32_t>(at / item_ints);
          ++pl.walk_real_items;
        }
      }
    }
  pl.walk_ok = true;
}

// Appends to requested nodes since the plan was made (no fork, no prune): the lists stay as they
// are except for
//  * the valid count of each grown node's last page and the limits of its query tokens;
//  * pages the appends started (tree-walk lists only, and only if the plan holds no other lists):
//    an odd page of the node's run becomes page b of the node's last block, wherever that block
//    is listed; an even one opens a new block in the room behind the private blocks of the
//    wavefront that holds the node -- if the node is private to one wavefront of one row block,
//    is asked for by one request and room is left; else the caller plans afresh.
// A new block goes behind the wavefront's other blocks, not next to its node's; the kernel's
// result does not depend on the order of a wavefront's blocks beyond rounding.  Mask flags are left
// alone: a flag that a fresh plan would no longer set only costs the masked code path.
bool Planner::patch_lengths(const PageTable &pt, Plan *plan, std::vector<int32_t> *dev_patches) {
  Plan &pl = *plan;
  if (!pl.valid || pl.topology_version != pt.topology_version()) return false;
  const bool walk = pl.has_walk && pl.walk_ok;
  const bool new_pages = pl.structure_version != pt.structure_version();
  if (new_pages && (!walk || pl.has_split || pl.has_csr)) return false;
  const int32_t n_leaves = static_cast<int32_t>(pl.req_leaves.size());
  const int32_t N = pt.num_nodes(), P = pt.page_size();
  if (static_cast<int32_t>(stamp_.size()) < N) {
    stamp_.resize(N, 0);
    slot_.resize(N, 0);
  }
  if (stamp_next_ == std::numeric_limits<int32_t>::max()) {
    std::fill(stamp_.begin(), stamp_.end(), 0);
    stamp_next_ = 1;
  }
  const int32_t st = stamp_next_++;
  const bool had_patches = !dev_patches->empty();
  auto patch = [&](int32_t array, int64_t index, int32_t value) {
    dev_patches->push_back(array);
    dev_patches->push_back(static_cast<int32_t>(index));
    dev_patches->push_back(value);
  };
  const int32_t NW = pl.walk_waves, rb_ints = pl.rb_ints();
  for (int32_t i = 0; i < n_leaves; ++i) {
    const int32_t u = pl.req_leaves[i];
    const Node &nd = pt.node(u);
    const int32_t delta = nd.n_tokens - pl.req_tokens[i];
    if (delta == 0) continue;
    if (delta < 0 || nd.pages.empty()) return false;
    const int32_t ql = pl.req_q_lens.empty() ? 1 : pl.req_q_lens[i];
    const int32_t n_pages = static_cast<int32_t>(nd.pages.size());
    const int32_t new_valid = pt.page_valid(u, n_pages - 1);
    const int32_t q0 = pl.qoff[i];
    if (pl.qt_limit[q0 + ql - 1] + delta >= (1 << 24)) return false;
    for (int32_t j = 0; j < ql; ++j) pl.qt_limit[q0 + j] += delta;
    pl.req_minlim[i] += delta;
    const bool first_visit = stamp_[u] != st;
    stamp_[u] = st;
    if (first_visit) pl.unique_tokens += delta;
    if (pl.has_csr) pl.leaf_valid[pl.leaf_indptr[i + 1] - 1] = new_valid;
    if (pl.has_split) {
      const int32_t pg = pl.req_split_pg[i];
      if (pg < 0) return false;
      pl.pg_valid[pg] = new_valid;
      pl.pg_rec[2 * pg + 1] = (pl.pg_pos[pg] << 7) | new_valid;
      if (first_visit) {
        patch(kPatchPgRec, 2 * static_cast<int64_t>(pg) + 1, pl.pg_rec[2 * pg + 1]);
        (pl.req_in_group[i] ? pl.prefix_tokens : pl.suffix_tokens) += delta;
      }
      for (int32_t e = pl.req_qtpos_indptr[i]; e < pl.req_qtpos_indptr[i + 1]; ++e)
        for (int32_t j = 0; j < ql; ++j) {
          const int64_t at = 2 * static_cast<int64_t>(pl.req_qtpos[e] + j) + 1;
          pl.qt_rec[at] = pl.qt_limit[q0 + j];
          patch(kPatchQtRec, at, pl.qt_rec[at]);
        }
    }
    if (walk) {
      const int32_t e0 = pl.req_walk_blk_indptr[i], e1 = pl.req_walk_blk_indptr[i + 1];
      if (e0 == e1) return false;
      const int32_t old_pages = pl.req_pages[i];
      if (n_pages < old_pages || old_pages < 1) return false;
      if (n_pages > old_pages && !first_visit) return false;  // the node is asked for twice
      auto set_field = [&](int32_t blk, int slot, int32_t value) {
        pl.walk_blocks[static_cast<size_t>(blk) * Plan::kBlockInts + slot] = value;
        patch(kPatchWalkBlocks, static_cast<int64_t>(blk) * Plan::kBlockInts + slot, value);
      };
      // path position of the node's first token, from its last block: page a of that block is
      // page (old_pages - 1) & ~1 of the run
      const int32_t *last = &pl.walk_blocks[static_cast<size_t>(pl.req_walk_blk[e0]) * Plan::kBlockInts];
      const int32_t pos0 = (last[1] >> 7) - ((old_pages - 1) & ~1) * P;
      for (int32_t pi = old_pages - 1; pi < n_pages; ++pi) {
        const int32_t valid = pt.page_valid(u, pi), pos = pos0 + pi * P;
        if ((pi & 1) || pi == old_pages - 1) {
          // the page is (or becomes) page a or b of the node's last block, in every list
          for (int32_t e = e0; e < e1; ++e) {
            const int32_t blk = pl.req_walk_blk[e];
            if (pi & 1) {
              set_field(blk, 2, nd.pages[pi]);
              set_field(blk, 3, (pos << 7) | valid);
            } else {
              set_field(blk, 1, (pos << 7) | valid);
            }
          }
          continue;
        }
        // a new block, in the room of the wavefront that holds the node
        const int32_t home = pl.req_walk_home[i];
        if (home < 0 || e1 - e0 != 1) return false;
        const int32_t rb = home / NW, w = home % NW;
        int32_t *rbr = &pl.walk_rb[static_cast<size_t>(rb) * rb_ints];
        const int32_t count = rbr[3 + w] & 0xffff, room = static_cast<int32_t>(static_cast<uint32_t>(rbr[3 + w]) >> 16);
        if (count >= room) return false;
        int32_t at = rbr[1] + rbr[2] + count;
        for (int32_t v = 0; v < w; ++v) at += static_cast<int32_t>(static_cast<uint32_t>(rbr[3 + v]) >> 16);
        const int32_t old_blk = pl.req_walk_blk[e0];
        const int32_t rows = pl.walk_blocks[static_cast<size_t>(old_blk) * Plan::kBlockInts + 4];
        const int32_t flags = 1 | (pl.walk_blocks[static_cast<size_t>(old_blk) * Plan::kBlockInts + 5] & 2);
        const int32_t rec[Plan::kBlockInts] = {nd.pages[pi], (pos << 7) | valid, nd.pages[pi], 0, rows, flags, 0, 0};
        for (int k = 0; k < Plan::kBlockInts; ++k) set_field(at, k, rec[k]);
        pl.req_walk_blk[e0] = at;
        rbr[3 + w] = (count + 1) | (room << 16);
        const int32_t item0 = pl.rb_item0[rb], item_ints = pl.item_ints();
        for (int32_t g = 0; g < pl.num_kv_heads; ++g) {
          const int64_t idx = static_cast<int64_t>(item0 + g) * item_ints + 3 + w;
          pl.walk_items[idx] = rbr[3 + w];
          patch(kPatchWalkItems, idx, rbr[3 + w]);
        }
        ++pl.walk_block_visits;
        pl.walk_max_item_blocks = std::max(pl.walk_max_item_blocks, rbr[2] + count + 1);
      }
      pl.req_pages[i] = n_pages;
      for (int32_t j = 0; j < ql; ++j) {
        const int64_t at = 2 * static_cast<int64_t>(pl.req_walk_qt[i] + j) + 1;
        pl.walk_qt[at] = pl.qt_limit[q0 + j];
        patch(kPatchWalkQt, at, pl.walk_qt[at]);
      }
    }
    pl.req_tokens[i] = nd.n_tokens;
  }
  if (new_pages || had_patches) {
    // The device applies a batch of patches in no particular order, so an index may appear only
    // once: keep the last value written to each (a wavefront's block count rises once per block
    // started, a block opened and then given its page b has two fields written twice; patches
    // that were already waiting in the list are older values of the same indices).
    std::vector<int32_t> &dp = *dev_patches;
    std::unordered_set<int64_t> seen;
    seen.reserve(dp.size() / 3);
    size_t keep = dp.size();
    const size_t first_patch = 0;  // the whole list is one batch
    for (size_t k = dp.size(); k > first_patch; k -= 3) {
      const int64_t key = (static_cast<int64_t>(dp[k - 3]) << 40) | static_cast<uint32_t>(dp[k - 2]);
      if (!seen.insert(key).second) continue;
      keep -= 3;
      dp[keep] = dp[k - 3];
      dp[keep + 1] = dp[k - 2];
      dp[keep + 2] = dp[k - 1];
    }
    dp.erase(dp.begin() + static_cast<std::ptrdiff_t>(first_patch), dp.begin() + static_cast<std::ptrdiff_t>(keep));
  }
  pl.table_version = pt.version();
  pl.structure_version = pt.structure_version();
  return true;
}

}  // namespace spex
