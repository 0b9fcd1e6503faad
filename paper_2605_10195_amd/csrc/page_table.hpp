// Host-side tree page table: node -> (parent, children, token count, page run) plus the
// stack allocator.  Integer bookkeeping only; no device code.
//
// A node is the state reached by one reasoning step, i.e. a run of tokens (paper Sec. 2.1).
// It owns the pages of its own tokens and reaches its prefix through the parent link, which
// is how sibling branches share prefix KV (Sec. 3.2, Sec. 4.3) without copies or refcounts:
// a child's first token always starts a fresh page, so a page belongs to exactly one node.
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

namespace spex {

constexpr int32_t kNoNode = -1;

struct Node {
  int32_t parent = kNoNode;
  int32_t n_tokens = 0;
  int32_t n_live_children = 0;
  bool alive = true;
  std::vector<int32_t> children;  // creation order, pruned ones included
  std::vector<int32_t> pages;     // page run in token order
};

class PageTable {
 public:
  PageTable(int64_t num_pages, int32_t page_size, const int32_t *free_order);

  int32_t page_size() const { return page_size_; }
  int64_t num_pages() const { return num_pages_; }
  int32_t num_nodes() const { return static_cast<int32_t>(nodes_.size()); }
  bool valid(int32_t u) const { return u >= 0 && u < num_nodes() && nodes_[u].alive; }
  const Node &node(int32_t u) const { return nodes_[u]; }
  uint64_t version() const { return version_; }
  // Bumped by fork, prune and every append that starts a new page; appends that only fill up a
  // node's last page leave it unchanged.
  uint64_t structure_version() const { return structure_version_; }
  // Bumped by fork and prune only: which nodes exist and who their parents are.
  uint64_t topology_version() const { return topology_version_; }

  // Creates n children under parent (kNoNode: roots); returns the first new id.
  int32_t fork(int32_t parent, int32_t n);
  // Pages an append of n_tokens would newly start.
  int32_t new_pages_needed(int32_t u, int32_t n_tokens) const;
  // Appends n_tokens; returns false (and changes nothing) if the pool is too small.
  // first_new receives the index, within the node's page run, of the first newly started page.
  bool append(int32_t u, int32_t n_tokens, int32_t *first_new);
  // Removes the subtree of u: pre-order, children in creation order, pages in run order,
  // each pushed on the free stack.
  void prune(int32_t u);

  int64_t live_nodes() const { return live_nodes_; }
  int64_t free_pages() const { return static_cast<int64_t>(free_.size()); }
  int64_t used_pages() const { return num_pages_ - free_pages(); }
  // Free stack, next page to be handed out first.
  std::vector<int32_t> free_list() const { return {free_.rbegin(), free_.rend()}; }

  // Valid tokens in page i of node u's run.
  int32_t page_valid(int32_t u, int32_t i) const {
    const int32_t left = nodes_[u].n_tokens - i * page_size_;
    return left < page_size_ ? left : page_size_;
  }

 private:
  int64_t num_pages_;
  int32_t page_size_;
  std::vector<Node> nodes_;
  std::vector<int32_t> free_;  // stack, top = back()
  int64_t live_nodes_ = 0;
  uint64_t version_ = 1;       // bumped by every mutation; the planner's cache key
  uint64_t structure_version_ = 1;
  uint64_t topology_version_ = 1;
};

}  // namespace spex
