/* CPU oracle for tree decode attention, plain C -- TEST INFRASTRUCTURE, not a product path.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may build or call this
 * file; the HIP library never does and shares nothing with it.
 *
 * What is computed: the same plain definition as oracle/tree_attention.py, written as loops so
 * that the benchmark-sized trees can be checked on every output row.  The paper (Sec. 3.2,
 * Sec. 4.1 insight 2, Sec. 4.3) fixes only that sibling branches reuse the KV cache of their
 * common prefix; a prefix-sharing scheme must give each branch what it would compute alone, so
 * for every requested node
 *   1. materialise: copy the K and V pieces of its root-to-node path, in path order, into one
 *      contiguous array [T][Hkv][D] (fp64, already decoded by the Python side);
 *   2. for query i of its q_len queries and query head h (kv head g = h / (Hq / Hkv)):
 *        visible(t):  t < T - q_len + 1 + i                                  (causal chain), or
 *                     t < T - q_len, or bit (t - (T - q_len)) of mask[i] set (draft token tree,
 *                                                                             Sec. 6.5)
 *        s_t = sm_scale * sum_d q[d] K[t][g][d]        over the visible t
 *        m = max s_t,  Z = sum exp(s_t - m),  out[d] = sum exp(s_t - m) V[t][g][d] / Z,
 *        lse = m + ln Z
 *      in double precision; the sums over t run in index order, the dot product over d may be
 *      summed in vector lanes (its rounding order is not fixed).
 * No blocking, no online softmax, no reuse between branches.  Requested nodes are independent,
 * so they are spread over threads; every output element is computed by one thread in the order
 * above, and the result does not depend on the number of threads.
 *
 * Pins (tests/test_oracle_pins.py): the hand-derived closed forms of
 * tests/golden/closed_form_cases.txt, nested Python loops over an independently materialised
 * branch, torch's fp64 scaled_dot_product_attention, draft-mask brute force, and agreement with
 * the numpy oracle on random trees.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
static double now(void) { return omp_get_wtime(); }
#else
#include <time.h>
static double now(void) {
  struct timespec ts;
  clock_gettime(CLOCK_MONOTONIC, &ts);
  return (double)ts.tv_sec + 1e-9 * (double)ts.tv_nsec;
}
#endif

/* Attention of one requested node over its materialised path.  K, V: [T][Hkv][D]; q: [q_len][Hq][D];
 * mask: q_len words or NULL; s: (Hq / Hkv) * T doubles, mrow / zrow: Hq / Hkv doubles of scratch.
 * Returns 0, or 1 if a query sees no token. */
static int branch_attention(const double *K, const double *V, int64_t T, int Hq, int Hkv, int D,
                            const double *q, int q_len, const uint32_t *mask, double sm_scale,
                            double *out, double *lse, double *s, double *mrow, double *zrow,
                            unsigned char *vis) {
  const int G = Hq / Hkv;
  const int64_t base = T - q_len; /* path position of draft 0 */
  for (int i = 0; i < q_len; ++i) {
    int64_t n_vis = 0;
    for (int64_t t = 0; t < T; ++t) {
      int v;
      if (mask == NULL)
        v = t < base + 1 + i;
      else
        v = t < base || ((mask[i] >> (t - base)) & 1u);
      vis[t] = (unsigned char)v;
      n_vis += v;
    }
    if (n_vis == 0) return 1;
    /* the G query heads of a kv head are taken together, so that a K or V row is fetched once */
    for (int g = 0; g < Hkv; ++g) {
      for (int hh = 0; hh < G; ++hh) mrow[hh] = -INFINITY;
      for (int64_t t = 0; t < T; ++t) {
        if (!vis[t]) continue;
        const double *k = K + (t * Hkv + g) * D;
        for (int hh = 0; hh < G; ++hh) {
          const double *qv = q + ((int64_t)i * Hq + g * G + hh) * D;
          double dot = 0.0;
#pragma omp simd reduction(+ : dot)
          for (int d = 0; d < D; ++d) dot += qv[d] * k[d];
          const double st = sm_scale * dot;
          s[(int64_t)hh * T + t] = st;
          if (st > mrow[hh]) mrow[hh] = st;
        }
      }
      for (int hh = 0; hh < G; ++hh) {
        double *o = out + ((int64_t)i * Hq + g * G + hh) * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        zrow[hh] = 0.0;
      }
      for (int64_t t = 0; t < T; ++t) {
        if (!vis[t]) continue;
        const double *v = V + (t * Hkv + g) * D;
        for (int hh = 0; hh < G; ++hh) {
          double *o = out + ((int64_t)i * Hq + g * G + hh) * D;
          const double w = exp(s[(int64_t)hh * T + t] - mrow[hh]);
          zrow[hh] += w;
          for (int d = 0; d < D; ++d) o[d] += w * v[d];
        }
      }
      for (int hh = 0; hh < G; ++hh) {
        double *o = out + ((int64_t)i * Hq + g * G + hh) * D;
        for (int d = 0; d < D; ++d) o[d] /= zrow[hh];
        lse[(int64_t)i * Hq + g * G + hh] = mrow[hh] + log(zrow[hh]);
      }
    }
  }
  return 0;
}

/* All requested nodes.
 *   piece_indptr [n_leaves + 1]: the pieces of leaf j, in path order, are piece_indptr[j] ..
 *   k_pieces / v_pieces [n_pieces]: HOST pointers to fp64 arrays [piece_tokens][Hkv][D]
 *   piece_tokens [n_pieces]
 *   q_lens [n_leaves]; q_off [n_leaves]: first query row of each leaf in q / out / lse
 *   q [rows][Hq][D], out [rows][Hq][D], lse [rows][Hq]; masks [rows] or NULL
 *   n_threads: 0 = the OpenMP default
 *   seconds[2]: thread-seconds spent materialising and in attention, summed over threads
 * Returns 0; -1 for bad arguments; 1 + j if leaf j has q_len < 1, q_len > T, a mask bit beyond
 * its drafts or a query that sees nothing; -2 if memory ran out.  threads_used receives the
 * number of threads that took part. */
int spex_oracle_attention(int32_t n_leaves, const int64_t *piece_indptr, const double *const *k_pieces,
                          const double *const *v_pieces, const int64_t *piece_tokens,
                          const int32_t *q_lens, const int64_t *q_off, const double *q,
                          const uint32_t *masks, int32_t Hq, int32_t Hkv, int32_t D, double sm_scale,
                          double *out, double *lse, int32_t n_threads, double *seconds,
                          int32_t *threads_used) {
  if (n_leaves < 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv != 0) return -1;
  int status = 0;
  double t_mat = 0.0, t_att = 0.0;
  int used = 1;
#ifdef _OPENMP
  if (n_threads > 0) omp_set_num_threads(n_threads);
#pragma omp parallel reduction(+ : t_mat, t_att)
#endif
  {
#ifdef _OPENMP
#pragma omp single
    used = omp_get_num_threads();
#pragma omp for schedule(dynamic, 1)
#endif
    for (int32_t j = 0; j < n_leaves; ++j) {
      int bad = 0;
#ifdef _OPENMP
#pragma omp atomic read
#endif
      bad = status;
      if (bad) continue;
      int64_t T = 0;
      for (int64_t p = piece_indptr[j]; p < piece_indptr[j + 1]; ++p) T += piece_tokens[p];
      const int ql = q_lens[j];
      int err = 0;
      if (ql < 1 || ql > T) err = 1 + j;
      if (!err && masks)
        for (int i = 0; i < ql; ++i)
          if (ql < 32 && (masks[q_off[j] + i] >> ql)) err = 1 + j;
      double *K = NULL, *V = NULL, *s = NULL, *mz = NULL;
      const int G = Hq / Hkv;
      unsigned char *vis = NULL;
      if (!err) {
        const size_t row = (size_t)Hkv * (size_t)D;
        K = (double *)malloc(sizeof(double) * row * (size_t)T);
        V = (double *)malloc(sizeof(double) * row * (size_t)T);
        s = (double *)malloc(sizeof(double) * (size_t)T * (size_t)G);
        mz = (double *)malloc(sizeof(double) * 2 * (size_t)G);
        vis = (unsigned char *)malloc((size_t)T);
        if (!K || !V || !s || !mz || !vis) err = -2;
      }
      if (!err) {
        const double t0 = now();
        const size_t row = (size_t)Hkv * (size_t)D;
        size_t at = 0;
        for (int64_t p = piece_indptr[j]; p < piece_indptr[j + 1]; ++p) {
          const size_t n = (size_t)piece_tokens[p] * row;
          memcpy(K + at, k_pieces[p], sizeof(double) * n);
          memcpy(V + at, v_pieces[p], sizeof(double) * n);
          at += n;
        }
        const double t1 = now();
        const int r = branch_attention(K, V, T, Hq, Hkv, D, q + q_off[j] * Hq * D, ql,
                                       masks ? masks + q_off[j] : NULL, sm_scale,
                                       out + q_off[j] * Hq * D, lse + q_off[j] * Hq, s, mz, mz + G, vis);
        const double t2 = now();
        t_mat += t1 - t0;
        t_att += t2 - t1;
        if (r) err = 1 + j;
      }
      free(K);
      free(V);
      free(s);
      free(mz);
      free(vis);
      if (err) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
        status = err;
      }
    }
  }
  if (seconds) {
    seconds[0] = t_mat;
    seconds[1] = t_att;
  }
  if (threads_used) *threads_used = used;
  return status;
}
