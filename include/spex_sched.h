/*
 * spex_sched.h -- host-side scheduling primitives of speculative Tree-of-Thought exploration.
 *
 * The decisions that shape the search tree whose KV cache spex_tree.h serves: how many children
 * a frontier node gets (BFS / REBASE widths, Sec. 2.1.1), which node a tree search visits next
 * (UCB, Sec. 2.1.2) and which nodes it will visit in its next k iterations (speculative selection
 * for DFS, Sec. 4.2, Alg. 1), how a global speculative budget is split over queries (Sec. 4.3,
 * Eq. 1-2) and when a query may stop (Sec. 4.4, Eq. 3-4).  They run between kernel launches on
 * the CPU; every pointer is a HOST pointer owned by the caller, nothing is allocated that outlives
 * the call, no GPU is touched.  All arithmetic is IEEE binary64 in the order stated, so that an
 * independent implementation reproduces every integer result; sums run in index order.
 *
 * Status codes are spex_status_t (spex_tree.h): SPEX_OK or SPEX_ERR_INVALID_ARG (null pointer,
 * negative count, non-finite or out-of-range parameter as stated per call); on error no output is
 * written.
 */
#ifndef SPEX_SCHED_H_
#define SPEX_SCHED_H_

#include <stdint.h>

#include "spex_tree.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * BFS expansion widths (Sec. 2.1.1, the REBASE rule): with budget B_i at the current depth and
 * balance temperature T_b > 0,
 *     W_j = Round( B_i * exp(R_j / T_b) / sum_k exp(R_k / T_b) )
 * evaluated as e_j = exp((R_j - max_k R_k) / T_b), s = e_0 + e_1 + ..., W_j = Round(B_i * (e_j / s)),
 * Round = nearest integer, halves to the even one.  The widths need not add up to B_i.
 *   rewards[n] finite, budget >= 0, widths[n] out.  n == 0 is allowed.
 * The same rule distributes the BFS speculative budget (= number of nodes that have finished
 * their step) over those finished nodes (Sec. 4.2, "Speculation for Breadth-First Search").
 */
spex_status_t spex_sched_rebase_widths(const double *rewards, int32_t n, int32_t budget,
                                       double temperature, int32_t *widths);

/*
 * Search tree of a DFS / MCTS query as parallel arrays over n_nodes nodes; node 0 is the root,
 * parent[u] < u for u > 0 (parent[0] = -1), children are visited in index order.
 *   visits[u]    N: how often the node was on a selected path (>= 0)
 *   value_sum[u] sum of the rewards backed up through the node; Q = value_sum / visits (0 if
 *                visits == 0)
 *   state[u]     SPEX_NODE_PLAIN, SPEX_NODE_ACTIVE (under expansion, primary or speculative) or
 *                SPEX_NODE_SPEC_DONE (expanded speculatively; spec_reward[u] holds its reward)
 */
enum { SPEX_NODE_PLAIN = 0, SPEX_NODE_ACTIVE = 1, SPEX_NODE_SPEC_DONE = 2 };
typedef struct {
  int32_t n_nodes;
  const int32_t *parent;
  const int64_t *visits;
  const double *value_sum;
  const int32_t *state;
  const double *spec_reward;
  double c; /* exploration constant of UCB, >= 0 */
} spex_search_tree_t;

/*
 * One UCB descent (Sec. 2.1.2): starting at the root, while the node has children move to the
 * child a that maximises  Q(a) + c * sqrt(ln N(s) / N(a)),  s the current node; a child with
 * N(a) == 0 counts as +infinity, ties go to the lowest index, ln N(s) is taken as 0 when
 * N(s) == 0.  *selected = the childless node reached.
 */
spex_status_t spex_sched_ucb_select(const spex_search_tree_t *tree, int32_t *selected);

/*
 * Speculative selection for DFS (Sec. 4.2, Alg. 1): the nodes the search is predicted to select
 * in its next k iterations, most likely first.  Works on a private copy of (visits, value_sum):
 *   repeat until k nodes are selected:
 *     node = UCB descent on the copy (as spex_sched_ucb_select)
 *     node is SPEC_DONE: its stored reward is backed up on the copy along the root path
 *         (visits += 1, value_sum += spec_reward[node] for the node and all its ancestors) and
 *         the descent is repeated;
 *     node is ACTIVE, or was selected earlier in this call: it is skipped -- a visit without
 *         reward is counted along its root path (visits += 1) and the descent is repeated;
 *     otherwise node is appended to the result and a visit is counted along its root path, so
 *         that the next descent is conditioned on this choice.
 * Readings: the algorithm as printed repeats the descent on an unchanged tree after a skip, which
 * would return the same node; counting a visit is what moves UCB on.  The call gives up after
 * k + 4 * n_nodes descents (a guard for trees whose every childless node is taken) and returns
 * what it has.  selected[k] out, *n_selected <= k.  k >= 0.
 */
spex_status_t spex_sched_dfs_speculate(const spex_search_tree_t *tree, int32_t k, int32_t *selected,
                                       int32_t *n_selected);

/*
 * Inter-query budget allocation (Sec. 4.3, Eq. 1-2).  For query q with parallel capacity C_q
 * (capacity[q] >= 0), predicted hit rate P_q (hit_rate[q] in [0, 1]) and reusable KV state
 * S_KV(q) (kv_bytes[q] >= 0; see spex_tree_path_kv_bytes), and model parameter size S_w >= 0:
 *     score_q = C_q * P_q * (S_w + S_KV(q))                                   (Eq. 1)
 *     k_q = min( C_q, floor( k_total * exp(tau * score_q) / sum_q' exp(tau * score_q') ) )   (Eq. 2)
 * evaluated as z_q = tau * score_q, e_q = exp(z_q - max z), s = e_0 + e_1 + ..., floor(k_total * (e_q / s)).
 * tau finite, k_total >= 0.  k[n] out; scores[n] out or NULL.
 */
spex_status_t spex_sched_allocate_budget(const int32_t *capacity, const double *hit_rate,
                                         const double *kv_bytes, int32_t n, double param_bytes,
                                         double tau, int32_t k_total, int32_t *k, double *scores);

/*
 * S_KV(q) of Eq. 1 read from the page table: bytes of K and V held by the tokens on the
 * root-to-node path of `node` (tokens * 2 * num_kv_heads * head_dim * element size; fp8: plus
 * 8 * num_kv_heads bytes of scales for every page on the path), i.e. the cache every branch
 * forked below `node` reuses instead of recomputing.  SPEX_ERR_BAD_NODE for an unknown or pruned
 * node.  HOST call, no GPU work.
 */
spex_status_t spex_tree_path_kv_bytes(const spex_tree_t *tree, spex_node_t node, double *bytes);

/*
 * Early termination for skewed trees (Sec. 4.4, Eq. 3-4).  n answers so far, answer_id[i] names
 * the hypothesis answer i belongs to (any int32), weight[i] >= 0 its reward.  conf(h) = sum of the
 * weights of h's answers (index order); 1st and 2nd = the hypotheses with the largest and second
 * largest conf (ties: the smaller id first).
 *     terminate  iff  n >= t  and  conf_1st - conf_2nd > alpha * avg(w_2nd),
 * avg(w_2nd) = conf_2nd / (number of answers of the 2nd hypothesis); with a single hypothesis
 * conf_2nd and avg(w_2nd) are 0.  No answers: never terminate.
 *   *terminate out (0 / 1); *best out or NULL: id of the 1st hypothesis (0 if n == 0).
 */
spex_status_t spex_sched_early_termination(const int32_t *answer_id, const double *weight, int32_t n,
                                           int32_t t, double alpha, int32_t *terminate,
                                           int32_t *best);

#ifdef __cplusplus
}
#endif
#endif /* SPEX_SCHED_H_ */
