// Per-launch planner: flattens parent links of the requested nodes into root-to-node page
// lists (CSR), shared-prefix groups, private suffixes, split chunks ("tasks"), the partial-result
// slots each task writes and the merge list of every query token.  Host integer work only.
//
// Rules (they fix the result uniquely, so that it can be compared bit for bit with an
// independent model):
//  * query tokens are numbered leaf-major; query token (leaf, i) sees T - q_len + 1 + i positions;
//  * live[u] = number of requested nodes in u's subtree, u included;
//  * group  = node on a requested path with live >= 2 and >= 1 token; ascending node id;
//             rows = query tokens of all requested nodes below it, in request order;
//  * suffix = maximal tail of a requested node's path with live == 1, root side first;
//  * a segment of n pages is cut into c = ceil(n / chunk_pages) chunks, chunk j = pages
//    [j*n/c, (j+1)*n/c);
//  * tasks: group chunks first (group order, chunk order), then suffix chunks (request order,
//    chunk order); a task owns rows*Hkv partial slots from pbase (running sum), slot of
//    (kv head g, local query token r, head-in-group hh) = pbase + g*rows + r*G + hh;
//  * flag bit 0 (masked): a page of the task is partial, or a row's limit is smaller than the
//    path position following the task's last token;
//  * flag bit 1 (final): suffix task that is the only chunk of its suffix; the suffix kernel
//    folds the other pieces of its rows into it and writes the output rows itself;
//  * merge_qt: ascending query tokens that still go through the merge kernel (requested nodes
//    whose suffix is empty or has several chunks).
#pragma once

#include <cstdint>
#include <vector>

#include "page_table.hpp"

namespace spex {

struct Plan {
  // ---- cache key
  std::vector<int32_t> req_leaves, req_q_lens;
  uint64_t table_version = 0;
  int32_t req_prefix_chunk = -1, req_suffix_chunk = -1;
  bool valid = false;

  // ---- canonical arrays (see spex_plan_view_t)
  std::vector<int32_t> leaf_indptr, leaf_pages, leaf_valid, qt_limit, group_node;
  std::vector<int32_t> task_pg_begin, task_pg_count, task_qt_begin, task_qt_count, task_pbase,
      task_flags;
  std::vector<int32_t> pg_id, pg_valid, pg_pos, qt_list;
  std::vector<int32_t> part_indptr, part_base, part_hstride, merge_qt;
  int32_t n_prefix_tasks = 0;
  int64_t n_partial_rows = 0;
  int32_t prefix_chunk_pages = 0, suffix_chunk_pages = 0;  // values used

  // ---- launch lists (device side).  A work item is kItemInts ints:
  //   {pg_begin, pg_count, qt_begin, qt_count, pbase, flags, kv_head, first_row}
  // pg_rec: per page entry {page id, path position << 7 | valid tokens};
  // qt_rec: per qt_list entry {query token, its limit}.
  static constexpr int kItemInts = 8;
  std::vector<int32_t> prefix_items, suffix_items, pg_rec, qt_rec;
  std::vector<int32_t> coop_items[3];  // cooperative shared-prefix kernel, 64 / 128 / 256 rows per workgroup
  int32_t prefix_row_tiles = 1, suffix_row_tiles = 1;  // 16-row MFMA tiles per wavefront
  int32_t max_rows_prefix = 0, max_rows_suffix = 0;
  int64_t prefix_tokens = 0, suffix_tokens = 0;        // distinct KV tokens per kind
};

enum class PlanError { kOk, kBadNode, kEmptyPath, kInvalid, kTooLarge };

class Planner {
 public:
  PlanError build(const PageTable &pt, const int32_t *leaves, const int32_t *q_lens,
                  int32_t n_leaves, int32_t num_q_heads, int32_t num_kv_heads,
                  int32_t prefix_chunk_pages, int32_t suffix_chunk_pages, Plan *plan);

 private:
  // dense per-node scratch, reset through touched_
  std::vector<int32_t> live_, pos0_, gindex_, touched_;
};

}  // namespace spex
