// Host-only fuzz of the planner and page table, built with AddressSanitizer and UBSan by
// test_host_sanitizers.py: random trees and requests, fresh tree-walk lists, then rounds of appends
// that are patched into the lists (or planned afresh when that is not possible).  After every
// round the lists must make every row read every page of its path exactly once, with the right
// position and length; unused room must be zero; a batch of patches must not give one list entry
// two different values.
#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <set>
#include <vector>

#include "../paper_2605_10195_amd/csrc/planner.hpp"

using namespace spex;

// what every row of the walk lists reads: (request -> multiset of (page, pos, valid))
static bool check_cover(const PageTable &pt, const Plan &pl, int G) {
  const int NW = pl.walk_waves, C = 16 * pl.walk_row_tiles, rb_ints = pl.rb_ints();
  const size_t n_rb = pl.walk_rb.size() / rb_ints;
  for (size_t rb = 0; rb < n_rb; ++rb) {
    const int32_t *r = &pl.walk_rb[rb * rb_ints];
    // rows -> query token
    std::map<int, int> row_tok;
    for (int w = 0; w < NW; ++w)
      for (int e = 0; e < r[3 + 2 * NW + w]; ++e)
        for (int h = 0; h < G; ++h) row_tok[w * C + e * G + h] = pl.walk_qt[2 * (r[3 + NW + w] + e)];
    std::map<int, std::multiset<std::vector<int>>> got;
    int b0 = r[1];
    auto scan = [&](int a, int b) {
      for (int k = a; k < b; ++k) {
        const int32_t *blk = &pl.walk_blocks[static_cast<size_t>(k) * 8];
        const int lo = blk[4] & 0xffff, hi = blk[4] >> 16;
        for (auto &rt : row_tok)
          if (rt.first >= lo && rt.first < hi) {
            got[rt.first].insert({blk[0], blk[1] >> 7, blk[1] & 127});
            if (blk[3]) got[rt.first].insert({blk[2], blk[3] >> 7, blk[3] & 127});
          }
      }
    };
    scan(b0, b0 + r[2]);
    b0 += r[2];
    for (int w = 0; w < NW; ++w) {
      const int count = r[3 + w] & 0xffff, room = static_cast<uint32_t>(r[3 + w]) >> 16;
      if (room < count) return false;
      scan(b0, b0 + count);
      for (int k = b0 + count; k < b0 + room; ++k)
        for (int j = 0; j < 8; ++j)
          if (pl.walk_blocks[static_cast<size_t>(k) * 8 + j] != 0) return false;
      b0 += room;
    }
    for (auto &rt : row_tok) {
      // request of the token
      int req = 0;
      while (req + 1 < static_cast<int>(pl.qoff.size()) && pl.qoff[req + 1] <= rt.second) ++req;
      std::multiset<std::vector<int>> want;
      int pos = 0;
      for (int k = pl.path_indptr[req]; k < pl.path_indptr[req + 1]; ++k) {
        const int u = pl.path_nodes[k];
        const Node &nd = pt.node(u);
        for (size_t i = 0; i < nd.pages.size(); ++i) {
          const int v = pt.page_valid(u, static_cast<int>(i));
          if (v > 0) want.insert({nd.pages[i], pos, v});
          pos += v;
        }
      }
      if (got[rt.first] != want) return false;
    }
  }
  return true;
}

int main(int argc, char **argv) {
  const int seeds = argc > 1 ? std::atoi(argv[1]) : 200;
  long patched = 0, fresh = 0, pages_patched = 0;
  for (int seed = 0; seed < seeds; ++seed) {
    std::mt19937 rng(seed);
    auto rnd = [&](int a, int b) { return a + static_cast<int>(rng() % static_cast<unsigned>(b - a + 1)); };
    const int P = 16, Hkv = 1 << rnd(0, 2), G = rnd(1, 8), Hq = Hkv * G;
    PageTable pt(4096, P, nullptr);
    std::vector<int> nodes;
    const int n_roots = rnd(1, 3);
    const int first = pt.fork(kNoNode, n_roots);
    for (int i = 0; i < n_roots; ++i) { nodes.push_back(first + i); pt.append(first + i, rnd(1, 120), nullptr); }
    for (int op = 0; op < rnd(3, 25); ++op) {
      const int u = nodes[rng() % nodes.size()];
      if (!pt.valid(u) || pt.node(u).n_tokens == 0) continue;
      const int n = rnd(1, 4), f = pt.fork(u, n);
      for (int i = 0; i < n; ++i) { nodes.push_back(f + i); pt.append(f + i, rnd(1, 70), nullptr); }
    }
    std::vector<int32_t> leaves, q_lens;
    for (int u : nodes)
      if (pt.valid(u) && rng() % 3 != 0) { leaves.push_back(u); q_lens.push_back(rnd(1, 3)); }
    if (leaves.empty()) continue;
    if (rng() % 4 == 0) { leaves.push_back(leaves[0]); q_lens.push_back(1); }   // a node asked for twice
    Planner planner;
    Plan plan;
    const int ntw = (int[]){0, 1, 2, 4}[rng() % 4], nw = (int[]){0, 4, 8}[rng() % 3];
    auto make = [&]() {
      PlanError e = planner.begin(pt, leaves.data(), q_lens.data(), nullptr, static_cast<int>(leaves.size()), Hq, Hkv, 0, 0, ntw, nw, &plan);
      if (e != PlanError::kOk) return false;
      planner.ensure_walk(pt, &plan);
      if (seed % 3 == 0) {                      // the split lists and the page CSR as well
        planner.ensure_csr(pt, &plan);
        if (planner.ensure_split(pt, &plan) != PlanError::kOk) return false;
      }
      return plan.walk_ok;
    };
    if (!make()) continue;
    ++fresh;
    if (!check_cover(pt, plan, G)) { std::printf("seed %d: fresh plan does not cover\n", seed); return 1; }
    std::vector<int32_t> patches;
    for (int step = 0; step < 60; ++step) {
      bool started = false;
      for (size_t i = 0; i < leaves.size(); ++i) {
        const int u = leaves[i];
        if (pt.node(u).n_live_children > 0 || rng() % 2) continue;
        const int n = rnd(1, rng() % 8 == 0 ? 40 : 3);
        started |= pt.new_pages_needed(u, n) > 0;
        pt.append(u, n, nullptr);
      }
      patches.clear();
      if (planner.patch_lengths(pt, &plan, &patches)) {
        ++patched;
        pages_patched += started;
        std::map<std::pair<int, int>, int> seen;   // the same value twice is harmless
        for (size_t k = 0; k < patches.size(); k += 3) {
          auto it = seen.find({patches[k], patches[k + 1]});
          if (it != seen.end() && it->second != patches[k + 2]) { std::printf("seed %d: an index patched with two values\n", seed); return 1; }
          seen[{patches[k], patches[k + 1]}] = patches[k + 2];
        }
      } else {
        if (!make()) { std::printf("seed %d: replan failed\n", seed); return 1; }
        ++fresh;
      }
      if (!check_cover(pt, plan, G)) { std::printf("seed %d step %d: plan does not cover\n", seed, step); return 1; }
    }
  }
  std::printf("ok: %ld fresh plans, %ld patched (%ld of them with started pages)\n", fresh, patched, pages_patched);
  return 0;
}
