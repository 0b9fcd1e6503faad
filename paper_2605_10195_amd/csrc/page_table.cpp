#include "page_table.hpp"

namespace spex {

PageTable::PageTable(int64_t num_pages, int32_t page_size, const int32_t *free_order)
    : num_pages_(num_pages), page_size_(page_size) {
  free_.resize(static_cast<size_t>(num_pages));
  // free_order[0] must be popped first, so it goes to the back of the stack vector.
  for (int64_t i = 0; i < num_pages; ++i) {
    const int32_t page = free_order ? free_order[i] : static_cast<int32_t>(i);
    free_[static_cast<size_t>(num_pages - 1 - i)] = page;
  }
}

int32_t PageTable::fork(int32_t parent, int32_t n) {
  const int32_t first = num_nodes();
  nodes_.resize(nodes_.size() + static_cast<size_t>(n));
  for (int32_t i = 0; i < n; ++i) {
    nodes_[first + i].parent = parent;
    if (parent != kNoNode) nodes_[parent].children.push_back(first + i);
  }
  if (parent != kNoNode) nodes_[parent].n_live_children += n;
  live_nodes_ += n;
  ++version_;
  ++structure_version_;
  ++topology_version_;
  return first;
}

int32_t PageTable::new_pages_needed(int32_t u, int32_t n_tokens) const {
  const Node &nd = nodes_[u];
  const int64_t total = static_cast<int64_t>(nd.n_tokens) + n_tokens;
  const int64_t pages = (total + page_size_ - 1) / page_size_;
  return static_cast<int32_t>(pages - static_cast<int64_t>(nd.pages.size()));
}

bool PageTable::append(int32_t u, int32_t n_tokens, int32_t *first_new) {
  const int32_t need = new_pages_needed(u, n_tokens);
  if (need > free_pages()) return false;
  Node &nd = nodes_[u];
  if (first_new) *first_new = static_cast<int32_t>(nd.pages.size());
  for (int32_t i = 0; i < need; ++i) {
    nd.pages.push_back(free_.back());
    free_.pop_back();
  }
  nd.n_tokens += n_tokens;
  ++version_;
  if (need > 0) ++structure_version_;
  return true;
}

void PageTable::prune(int32_t u) {
  const int32_t parent = nodes_[u].parent;
  if (parent != kNoNode) --nodes_[parent].n_live_children;
  std::vector<int32_t> stack{u};
  while (!stack.empty()) {
    const int32_t w = stack.back();
    stack.pop_back();
    Node &nd = nodes_[w];
    if (!nd.alive) continue;
    nd.alive = false;
    --live_nodes_;
    for (int32_t p : nd.pages) free_.push_back(p);
    nd.pages.clear();
    nd.pages.shrink_to_fit();
    nd.n_live_children = 0;
    for (auto it = nd.children.rbegin(); it != nd.children.rend(); ++it) stack.push_back(*it);
  }
  ++version_;
  ++structure_version_;
  ++topology_version_;
}

}  // namespace spex
