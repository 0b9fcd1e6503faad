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
#include <utility>
#include <vector>

#include "page_table.hpp"

namespace spex {

struct Plan {
  // ---- cache key
  std::vector<int32_t> req_leaves, req_q_lens;
  std::vector<uint32_t> req_masks;  // draft visibility masks per query token, or empty (causal chain)
  uint64_t table_version = 0, structure_version = 0, topology_version = 0;
  int32_t req_prefix_chunk = -1, req_suffix_chunk = -1;
  int32_t num_q_heads = 0, num_kv_heads = 0;
  bool valid = false;
  // The lists are built in stages, each on first use: the page CSR (dump and tests only), the
  // split lists (shared-prefix / suffix / merge kernels) and the tree-walk lists.
  bool has_csr = false, has_split = false, has_walk = false;

  // ---- common to all stages
  std::vector<int32_t> path_indptr, path_nodes;  // root-to-node paths of the requests
  std::vector<int32_t> qoff;                     // first query token of each request
  std::vector<int32_t> req_tokens;               // tokens of each requested node when planned / patched
  int64_t unique_tokens = 0;                     // KV tokens on the requested paths, each node once
  // first path position that some query of the request does not see: T - q_len + (number of
  // leading drafts all its queries see); T - q_len + 1 for the causal chain
  std::vector<int32_t> req_minlim;
  std::vector<int32_t> qt_mask;                  // {index of the query in its request, mask} per query token; empty without masks
  // ---- where an append to a requested node shows up (see Planner::patch_lengths)
  std::vector<int32_t> req_split_pg, req_in_group, req_qtpos_indptr, req_qtpos;
  std::vector<int32_t> req_walk_blk_indptr, req_walk_blk, req_walk_qt;
  std::vector<int32_t> req_pages;      // pages of each requested node when planned / patched
  // row block * NW + wavefront whose private list alone holds the requested node's blocks, else -1
  std::vector<int32_t> req_walk_home;
  std::vector<int32_t> rb_item0;       // per row block: its work item for kv head 0 (the others follow)

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

  // ---- tree-walk lists (see the rules above build_walk in planner.cpp)
  bool walk_ok = false;         // every requested node's rows fit one wavefront
  int32_t walk_row_tiles = 0;   // 16-row tiles per wavefront (1, 2 or 4)
  int32_t walk_waves = 0;       // NW: wavefronts of rows per row block (2, 4 or 8; with 2 the kernel runs two wavefronts on each)
  int32_t req_walk_row_tiles = -1, req_walk_waves = -1;
  // row blocks: 3 + 3 * NW ints each
  //   {root node, first block, shared blocks, private blocks of wavefronts 0..NW-1 as
  //    count | room << 16 (room >= count block records are set aside for the wavefront, the
  //    unused ones zero), first walk_qt entry of wavefronts 0..NW-1, walk_qt entries of
  //    wavefronts 0..NW-1}
  int rb_ints() const { return 3 + 3 * walk_waves; }
  std::vector<int32_t> walk_rb;
  // blocks: kBlockInts ints each {page a, pos_a << 7 | valid_a, page b, pos_b << 7 | valid_b
  //   (0: no page b), first row | (last row + 1) << 16, flags (bit 0: token mask needed, bit 1:
  //   node shared with another row block), 0, 0}
  static constexpr int kBlockInts = 8;
  std::vector<int32_t> walk_blocks;
  std::vector<int32_t> walk_qt;     // {query token, limit} in row order
  // launch order: item_ints() = 16 (NW <= 4) or 32 (NW = 8) ints per workgroup {kv head, first
  //   block, shared blocks, private blocks[NW], walk_qt first[NW], walk_qt count[NW], zeros..,
  //   row block index in the last int}; a padding item has row block index -1 and no blocks
  int item_ints() const { return walk_waves <= 4 ? 16 : 32; }
  std::vector<int32_t> walk_items;
  int32_t walk_real_items = 0;       // workgroups with work
  int32_t walk_max_item_blocks = 0;  // longest workgroup: shared blocks + most private blocks of a wavefront
  int64_t walk_block_visits = 0;  // blocks over all row blocks (a block shared by two row blocks counts twice)
};

enum class PlanError { kOk, kBadNode, kEmptyPath, kInvalid, kTooLarge };

// Device arrays a length patch can touch; a patch is the triple {array, int index, new value}.
enum PatchArray : int32_t { kPatchPgRec = 0, kPatchQtRec = 1, kPatchWalkBlocks = 2, kPatchWalkQt = 3, kPatchWalkItems = 4 };

class Planner {
 public:
  // Validates the request, walks the paths and computes the limits; the lists follow on demand.
  PlanError begin(const PageTable &pt, const int32_t *leaves, const int32_t *q_lens,
                  const uint32_t *draft_masks, int32_t n_leaves, int32_t num_q_heads, int32_t num_kv_heads,
                  int32_t prefix_chunk_pages, int32_t suffix_chunk_pages, int32_t walk_row_tiles,
                  int32_t walk_waves, Plan *plan);
  void ensure_csr(const PageTable &pt, Plan *plan);
  PlanError ensure_split(const PageTable &pt, Plan *plan);
  void ensure_walk(const PageTable &pt, Plan *plan);
  // Brings a plan up to date after appends to requested nodes (no fork or prune since it was
  // made).  Tokens that fill up a last page change valid counts and limits; a newly started page
  // becomes page b of the node's last block or, in tree-walk lists that are the plan's only
  // lists, a new block in the room set aside behind its wavefront's private blocks.  Returns
  // false if that is not possible (the caller then plans afresh; the plan may be half changed).
  bool patch_lengths(const PageTable &pt, Plan *plan, std::vector<int32_t> *dev_patches);

 private:
  std::vector<int32_t> multi_, last_pg_;
  std::vector<int32_t> stamp_, slot_;  // per-node scratch of build_walk, valid where stamp_ == current stamp
  // scratch of the request ordering in ensure_walk: pre-order rank and child ranges per node,
  // (parent, child) edges of the requested paths, traversal stack, (rank, request) keys
  std::vector<int32_t> rank_, child_lo_, child_n_, dfs_;
  std::vector<std::pair<int32_t, int32_t>> edges_;
  std::vector<int64_t> keyed_;
  int32_t stamp_next_ = 1;
  // dense per-node scratch, reset through touched_
  std::vector<int32_t> live_, pos0_, gindex_, touched_;
};

}  // namespace spex
