// The C ABI's host side under AddressSanitizer, built by test_host_sanitizers.py with hipcc (host code
// instrumented, device code as in the product).  No GPU is needed: the pools are null, so appends
// only move the page table, and the plans are dumped instead of launched.  Random forks, appends,
// prunes, one-token appends to many nodes, plan dumps of both kinds, path and statistics reads.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>
#include "../include/spex_sched.h"
#include "../include/spex_tree.h"

int main(int argc, char **argv) {
  const int seeds = argc > 1 ? std::atoi(argv[1]) : 100;
  long calls = 0;
  for (int seed = 0; seed < seeds; ++seed) {
    std::mt19937 rng(seed);
    auto rnd = [&](int a, int b) { return a + static_cast<int>(rng() % static_cast<unsigned>(b - a + 1)); };
    spex_config_t cfg;
    std::memset(&cfg, 0, sizeof cfg);
    cfg.num_kv_heads = 1 << rnd(0, 3);
    cfg.num_q_heads = cfg.num_kv_heads * rnd(1, 8);
    cfg.head_dim = (int[]){64, 128, 96}[rng() % 3];
    cfg.page_size = 16;
    cfg.q_dtype = SPEX_BF16;
    cfg.kv_dtype = (rng() % 2) ? SPEX_BF16 : SPEX_FP8_E4M3;
    cfg.num_pages = rnd(64, 2048);
    spex_tree_t *t = nullptr;
    if (spex_tree_create(&cfg, &t) != SPEX_OK) { std::printf("seed %d: create failed\n", seed); return 1; }
    std::vector<spex_node_t> nodes;
    for (int op = 0; op < 120; ++op, ++calls) {
      const int what = static_cast<int>(rng() % 10);
      if (nodes.empty() || what == 0) {
        spex_node_t kids[4];
        const int n = rnd(1, 3);
        const spex_node_t parent = (nodes.empty() || rng() % 4 == 0) ? SPEX_NO_NODE : nodes[rng() % nodes.size()];
        if (spex_tree_fork(t, parent, n, kids) == SPEX_OK)
          for (int i = 0; i < n; ++i) nodes.push_back(kids[i]);
      } else if (what <= 3) {
        (void)spex_tree_append_step(t, nodes[rng() % nodes.size()], rnd(1, 60), nullptr, nullptr, nullptr, nullptr, nullptr);
      } else if (what == 4 && nodes.size() > 3) {
        (void)spex_tree_prune(t, nodes[rng() % nodes.size()]);
      } else if (what == 5) {
        std::vector<spex_node_t> some;
        for (spex_node_t u : nodes) if (rng() % 3 == 0) some.push_back(u);
        (void)spex_tree_append_tokens(t, some.data(), static_cast<int32_t>(some.size()), nullptr, nullptr, nullptr, nullptr, nullptr);
      } else {
        std::vector<spex_node_t> leaves;
        std::vector<int32_t> q_lens;
        for (spex_node_t u : nodes) if (rng() % 2) { leaves.push_back(u); q_lens.push_back(rnd(1, 5)); }
        spex_walk_view_t wv;
        spex_plan_view_t pv;
        (void)spex_tree_walk_dump(t, leaves.data(), q_lens.data(), nullptr, static_cast<int32_t>(leaves.size()), &wv);
        if (what >= 8) (void)spex_tree_plan_dump(t, leaves.data(), q_lens.data(), static_cast<int32_t>(leaves.size()), &pv);
        if (!leaves.empty()) {
          int32_t pages[64], valid[64], n = 0;
          (void)spex_tree_path_pages(t, leaves[0], pages, valid, 64, &n);
          double bytes = 0;
          (void)spex_tree_path_kv_bytes(t, leaves[0], &bytes);
        }
        int64_t a, b, c;
        (void)spex_tree_stats(t, &a, &b, &c);
      }
    }
    spex_tree_destroy(t);
  }
  std::printf("ok: %ld calls\n", calls);
  return 0;
}
