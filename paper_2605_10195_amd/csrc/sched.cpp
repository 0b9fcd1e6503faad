// Host-side scheduling primitives (spex_sched.h): REBASE widths (Sec. 2.1.1), UCB descent
// (Sec. 2.1.2), speculative selection for DFS (Sec. 4.2, Alg. 1), inter-query budget allocation
// (Sec. 4.3, Eq. 1-2) and early termination (Sec. 4.4, Eq. 3-4).  IEEE binary64 throughout, sums in
// index order, std::exp / std::log / std::sqrt; no GPU work.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <vector>

#include "../../include/spex_sched.h"

// every product and sum below is rounded on its own, as the header's evaluation order states
#pragma STDC FP_CONTRACT OFF

namespace {

// Children of every node in index order, CSR.
struct Children {
  std::vector<int32_t> indptr, list;
  explicit Children(const spex_search_tree_t &t) : indptr(t.n_nodes + 1, 0), list(t.n_nodes > 0 ? t.n_nodes - 1 : 0) {
    for (int32_t u = 1; u < t.n_nodes; ++u) ++indptr[t.parent[u] + 1];
    for (int32_t u = 0; u < t.n_nodes; ++u) indptr[u + 1] += indptr[u];
    std::vector<int32_t> fill(indptr.begin(), indptr.end() - 1);
    for (int32_t u = 1; u < t.n_nodes; ++u) list[fill[t.parent[u]]++] = u;
  }
};

bool tree_ok(const spex_search_tree_t *t) {
  if (!t || t->n_nodes < 1 || !t->parent || !t->visits || !t->value_sum || !t->state || !t->spec_reward)
    return false;
  if (!(t->c >= 0.0) || !std::isfinite(t->c)) return false;
  if (t->parent[0] != -1) return false;
  for (int32_t u = 0; u < t->n_nodes; ++u) {
    if (u > 0 && (t->parent[u] < 0 || t->parent[u] >= u)) return false;
    if (t->visits[u] < 0 || !std::isfinite(t->value_sum[u]) || !std::isfinite(t->spec_reward[u])) return false;
    if (t->state[u] != SPEX_NODE_PLAIN && t->state[u] != SPEX_NODE_ACTIVE && t->state[u] != SPEX_NODE_SPEC_DONE)
      return false;
  }
  return true;
}

// One descent: from the root to a childless node, each time to the child with the largest
// Q + c * sqrt(ln N(s) / N(a)); unvisited children first, lowest index on ties.
int32_t descend(const Children &ch, double c, const int64_t *visits, const double *value_sum) {
  int32_t s = 0;
  for (;;) {
    const int32_t a0 = ch.indptr[s], a1 = ch.indptr[s + 1];
    if (a0 == a1) return s;
    const double log_n = visits[s] > 0 ? std::log(static_cast<double>(visits[s])) : 0.0;
    int32_t best = -1;
    double best_score = 0.0;
    for (int32_t i = a0; i < a1; ++i) {
      const int32_t a = ch.list[i];
      double score;
      if (visits[a] == 0) {
        score = std::numeric_limits<double>::infinity();
      } else {
        const double n = static_cast<double>(visits[a]);
        score = value_sum[a] / n + c * std::sqrt(log_n / n);
      }
      if (best < 0 || score > best_score) {
        best = a;
        best_score = score;
      }
    }
    s = best;
  }
}

}  // namespace

extern "C" {

spex_status_t spex_sched_rebase_widths(const double *rewards, int32_t n, int32_t budget,
                                       double temperature, int32_t *widths) {
  if (n < 0 || budget < 0 || (n > 0 && (!rewards || !widths))) return SPEX_ERR_INVALID_ARG;
  if (!(temperature > 0.0) || !std::isfinite(temperature)) return SPEX_ERR_INVALID_ARG;
  for (int32_t j = 0; j < n; ++j)
    if (!std::isfinite(rewards[j])) return SPEX_ERR_INVALID_ARG;
  if (n == 0) return SPEX_OK;
  const double top = *std::max_element(rewards, rewards + n);
  std::vector<double> e(n);
  double s = 0.0;
  for (int32_t j = 0; j < n; ++j) {
    e[j] = std::exp((rewards[j] - top) / temperature);
    s += e[j];
  }
  // std::nearbyint rounds halves to even in the default rounding mode, which nothing here changes
  for (int32_t j = 0; j < n; ++j) widths[j] = static_cast<int32_t>(std::nearbyint(budget * (e[j] / s)));
  return SPEX_OK;
}

spex_status_t spex_sched_ucb_select(const spex_search_tree_t *tree, int32_t *selected) {
  if (!tree_ok(tree) || !selected) return SPEX_ERR_INVALID_ARG;
  const Children ch(*tree);
  *selected = descend(ch, tree->c, tree->visits, tree->value_sum);
  return SPEX_OK;
}

spex_status_t spex_sched_dfs_speculate(const spex_search_tree_t *tree, int32_t k, int32_t *selected,
                                       int32_t *n_selected) {
  if (!tree_ok(tree) || k < 0 || !n_selected || (k > 0 && !selected)) return SPEX_ERR_INVALID_ARG;
  const int32_t n = tree->n_nodes;
  const Children ch(*tree);
  std::vector<int64_t> visits(tree->visits, tree->visits + n);
  std::vector<double> value_sum(tree->value_sum, tree->value_sum + n);
  std::vector<char> taken(n, 0);
  std::vector<int32_t> out;
  out.reserve(k);
  const int64_t max_descents = static_cast<int64_t>(k) + 4 * static_cast<int64_t>(n);
  for (int64_t d = 0; d < max_descents && static_cast<int32_t>(out.size()) < k; ++d) {
    const int32_t node = descend(ch, tree->c, visits.data(), value_sum.data());
    double reward = 0.0;
    bool with_reward = false;
    if (tree->state[node] == SPEX_NODE_SPEC_DONE) {
      reward = tree->spec_reward[node];
      with_reward = true;
    } else if (tree->state[node] == SPEX_NODE_PLAIN && !taken[node]) {
      out.push_back(node);
      taken[node] = 1;
    }
    for (int32_t u = node; u >= 0; u = tree->parent[u]) {
      ++visits[u];
      if (with_reward) value_sum[u] += reward;
    }
  }
  std::copy(out.begin(), out.end(), selected);
  *n_selected = static_cast<int32_t>(out.size());
  return SPEX_OK;
}

spex_status_t spex_sched_allocate_budget(const int32_t *capacity, const double *hit_rate,
                                         const double *kv_bytes, int32_t n, double param_bytes,
                                         double tau, int32_t k_total, int32_t *k, double *scores) {
  if (n < 0 || k_total < 0 || (n > 0 && (!capacity || !hit_rate || !kv_bytes || !k)))
    return SPEX_ERR_INVALID_ARG;
  if (!std::isfinite(tau) || !(param_bytes >= 0.0) || !std::isfinite(param_bytes)) return SPEX_ERR_INVALID_ARG;
  for (int32_t q = 0; q < n; ++q)
    if (capacity[q] < 0 || !(hit_rate[q] >= 0.0 && hit_rate[q] <= 1.0) || !(kv_bytes[q] >= 0.0) ||
        !std::isfinite(kv_bytes[q]))
      return SPEX_ERR_INVALID_ARG;
  if (n == 0) return SPEX_OK;
  std::vector<double> z(n), e(n);
  for (int32_t q = 0; q < n; ++q) {
    const double score = capacity[q] * hit_rate[q] * (param_bytes + kv_bytes[q]);
    if (scores) scores[q] = score;
    z[q] = tau * score;
  }
  const double top = *std::max_element(z.begin(), z.end());
  double s = 0.0;
  for (int32_t q = 0; q < n; ++q) {
    e[q] = std::exp(z[q] - top);
    s += e[q];
  }
  for (int32_t q = 0; q < n; ++q) {
    const double share = std::floor(k_total * (e[q] / s));
    k[q] = std::min(capacity[q], static_cast<int32_t>(share));
  }
  return SPEX_OK;
}

spex_status_t spex_sched_early_termination(const int32_t *answer_id, const double *weight, int32_t n,
                                           int32_t t, double alpha, int32_t *terminate,
                                           int32_t *best) {
  if (n < 0 || !terminate || (n > 0 && (!answer_id || !weight)) || !std::isfinite(alpha))
    return SPEX_ERR_INVALID_ARG;
  for (int32_t i = 0; i < n; ++i)
    if (!(weight[i] >= 0.0) || !std::isfinite(weight[i])) return SPEX_ERR_INVALID_ARG;
  if (n == 0) {
    *terminate = 0;
    if (best) *best = 0;
    return SPEX_OK;
  }
  // hypotheses in order of first appearance; conf summed in answer order
  struct Hyp { int32_t id; double conf; int32_t count; };
  std::vector<Hyp> hyps;
  for (int32_t i = 0; i < n; ++i) {
    size_t h = 0;
    while (h < hyps.size() && hyps[h].id != answer_id[i]) ++h;
    if (h == hyps.size()) hyps.push_back({answer_id[i], 0.0, 0});
    hyps[h].conf += weight[i];
    ++hyps[h].count;
  }
  auto before = [](const Hyp &a, const Hyp &b) { return a.conf > b.conf || (a.conf == b.conf && a.id < b.id); };
  const Hyp *first = &hyps[0], *second = nullptr;
  for (const Hyp &h : hyps)
    if (before(h, *first)) first = &h;
  for (const Hyp &h : hyps)
    if (&h != first && (!second || before(h, *second))) second = &h;
  const double conf2 = second ? second->conf : 0.0;
  const double avg2 = second ? second->conf / second->count : 0.0;
  *terminate = (n >= t && first->conf - conf2 > alpha * avg2) ? 1 : 0;
  if (best) *best = first->id;
  return SPEX_OK;
}

}  // extern "C"
