// Host-only fuzz of the scheduling primitives (csrc/sched.cpp), built with AddressSanitizer and
// UBSan by test_host_sanitizers.py: random search trees and parameters, including empty and
// degenerate inputs; every output must stay inside the ranges the header promises.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <set>
#include <vector>

#include "../include/spex_sched.h"

int main(int argc, char **argv) {
  const int rounds = argc > 1 ? std::atoi(argv[1]) : 2000;
  std::mt19937 rng(12345);
  std::uniform_real_distribution<double> uni(0.0, 1.0);
  long selections = 0;
  for (int it = 0; it < rounds; ++it) {
    // ---- a random search tree
    const int n = 1 + static_cast<int>(rng() % 40);
    std::vector<int32_t> parent(n), state(n);
    std::vector<int64_t> visits(n);
    std::vector<double> value(n), spec(n);
    parent[0] = -1;
    for (int u = 0; u < n; ++u) {
      if (u > 0) parent[u] = static_cast<int32_t>(rng() % u);
      visits[u] = static_cast<int64_t>(rng() % 6);
      value[u] = visits[u] * uni(rng);
      state[u] = static_cast<int32_t>(rng() % 3);
      spec[u] = uni(rng);
    }
    spex_search_tree_t t{n, parent.data(), visits.data(), value.data(), state.data(), spec.data(), 2.0 * uni(rng)};
    int32_t sel = -7;
    if (spex_sched_ucb_select(&t, &sel) != SPEX_OK || sel < 0 || sel >= n) { std::printf("ucb: bad result\n"); return 1; }
    for (int u = 0; u < n; ++u)
      if (parent[u] == sel) { std::printf("ucb: the selected node has a child\n"); return 1; }
    const int k = static_cast<int>(rng() % 9);
    std::vector<int32_t> out(k > 0 ? k : 1, -1);
    int32_t n_out = -1;
    if (spex_sched_dfs_speculate(&t, k, out.data(), &n_out) != SPEX_OK || n_out < 0 || n_out > k) { std::printf("dfs: bad count\n"); return 1; }
    std::set<int32_t> distinct(out.begin(), out.begin() + n_out);
    if (static_cast<int>(distinct.size()) != n_out) { std::printf("dfs: a node selected twice\n"); return 1; }
    for (int32_t u : distinct)
      if (u < 0 || u >= n || state[u] != SPEX_NODE_PLAIN) { std::printf("dfs: bad node\n"); return 1; }
    selections += n_out;
    // ---- widths
    const int m = static_cast<int>(rng() % 20);
    std::vector<double> rewards(m > 0 ? m : 1);
    for (double &r : rewards) r = 4.0 * uni(rng) - 2.0;
    std::vector<int32_t> widths(m > 0 ? m : 1, -1);
    const int budget = static_cast<int>(rng() % 64);
    if (spex_sched_rebase_widths(rewards.data(), m, budget, 0.05 + uni(rng), widths.data()) != SPEX_OK) { std::printf("widths: error\n"); return 1; }
    for (int j = 0; j < m; ++j)
      if (widths[j] < 0 || widths[j] > budget) { std::printf("widths: out of range\n"); return 1; }
    // ---- budget allocation
    const int q = static_cast<int>(rng() % 12);
    std::vector<int32_t> cap(q > 0 ? q : 1), kq(q > 0 ? q : 1, -1);
    std::vector<double> hit(q > 0 ? q : 1), kvb(q > 0 ? q : 1), scores(q > 0 ? q : 1);
    for (int i = 0; i < q; ++i) { cap[i] = static_cast<int32_t>(rng() % 9); hit[i] = uni(rng); kvb[i] = 1e9 * uni(rng); }
    const int k_total = static_cast<int>(rng() % 100);
    if (spex_sched_allocate_budget(cap.data(), hit.data(), kvb.data(), q, 1.6e10, 1e-10 * uni(rng), k_total, kq.data(), scores.data()) != SPEX_OK) { std::printf("budget: error\n"); return 1; }
    long sum = 0;
    for (int i = 0; i < q; ++i) {
      if (kq[i] < 0 || kq[i] > cap[i]) { std::printf("budget: beyond a query's capacity\n"); return 1; }
      sum += kq[i];
    }
    if (sum > k_total) { std::printf("budget: more than the total\n"); return 1; }
    // ---- early termination
    const int a = static_cast<int>(rng() % 16);
    std::vector<int32_t> ans(a > 0 ? a : 1);
    std::vector<double> wt(a > 0 ? a : 1);
    for (int i = 0; i < a; ++i) { ans[i] = static_cast<int32_t>(rng() % 4); wt[i] = uni(rng); }
    int32_t term = -1, best = -1;
    if (spex_sched_early_termination(ans.data(), wt.data(), a, static_cast<int>(rng() % 8), uni(rng), &term, &best) != SPEX_OK || (term != 0 && term != 1)) { std::printf("termination: bad result\n"); return 1; }
    if (a > 0 && (best < 0 || best > 3)) { std::printf("termination: unknown answer\n"); return 1; }
    // ---- errors leave outputs alone
    int32_t keep = 1234;
    if (spex_sched_ucb_select(nullptr, &keep) != SPEX_ERR_INVALID_ARG || keep != 1234) { std::printf("ucb: error path\n"); return 1; }
    if (spex_sched_rebase_widths(rewards.data(), m, budget, 0.0, widths.data()) != SPEX_ERR_INVALID_ARG) { std::printf("widths: error path\n"); return 1; }
  }
  std::printf("ok: %ld speculative selections\n", selections);
  return 0;
}
