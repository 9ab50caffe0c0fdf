/*
 * CPU oracle for the fused star-join + model-prediction path and the
 * linear-algebra group-by aggregate.
 *
 * TEST INFRASTRUCTURE ONLY. This file is the slow, plain reference the GPU
 * library is checked against. Nothing in the product path may include, link
 * or call it, and it shares no code with the HIP sources.
 *
 * Everything is fp64 / int64. Inputs are the exact fp32 or bf16 values the
 * GPU sees, widened to double by the caller; nothing is rounded in here.
 *
 * What each function follows (paper: "Accelerating Machine Learning Queries
 * with Linear Algebra Query Processing", SSDBM 2023):
 *   lqo_join_predict   - Section 3.1 (star join of fact table A with its
 *                        dimension tables, result fed to a model) and the
 *                        first two lines of Eq. 1: T = sum_k I_k D_k M_k is
 *                        formed tuple by tuple, then predictions = T L.
 *                        I_k per the row-mapping definition of Section 2.3.3
 *                        (exactly one 1 per materialised row), so row i of
 *                        I_k D_k is row fk_k[i] of D_k.  M_k places the
 *                        columns of D_k side by side in T (Section 2.1).
 *   lqo_materialize    - the same T, returned instead of consumed.
 *   lqo_project_dims   - the underlined terms of Eq. 1: P_k = D_k M_k L,
 *                        i.e. D_k times the rows of L that belong to dim k.
 *   lqo_gather_sum     - the last line of Eq. 1: sum_k I_k P_k (plus the
 *                        fact table's own term).  Exists so that tests can
 *                        check Eq. 1's identity; the parity reference for
 *                        the GPU is lqo_join_predict.
 *   lqo_groupby_sum    - Section 2.2 (selection as a 0/1 vector), Section
 *                        2.3 (join as I), Section 2.4 (group mapping matrix
 *                        times a ones reduction vector; several grouping
 *                        columns as in Section 2.4.2), evaluated per tuple
 *                        with relational filter / join / GROUP BY / SUM
 *                        semantics.
 *
 * Readings taken where the paper is silent:
 *   - fact-table feature columns come first in T, then dimension 0, 1, ...
 *   - bias (optional) is added once per layer after the sum
 *   - a ReLU sits between layers, none after the last
 *   - a foreign key < 0 in the group-by drops the row (inner join)
 *   - group index is row-major over the grouping dimensions in dimension
 *     order (last grouping dimension fastest)
 *
 * Threading (nthreads > 1) splits fact rows into contiguous static chunks;
 * rows are independent in the predict path, and the group-by merges
 * per-thread int64 accumulators in thread order (integers: exact).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int clamp_threads(int nthreads) {
  if (nthreads < 1) return 1;
  return nthreads;
}

/* Number of threads the build can actually run (1 without OpenMP). */
int lqo_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Build the joined tuple of fact row i: [x_i | D_0[fk_0[i]] | ... ]. */
static void build_tuple(int64_t i, int32_t c_f, const double* X, int32_t K,
                        const int32_t* c, const double* const* D,
                        const int32_t* const* fk, double* t) {
  int64_t pos = 0;
  for (int32_t j = 0; j < c_f; ++j) t[pos++] = X[i * (int64_t)c_f + j];
  for (int32_t k = 0; k < K; ++k) {
    const double* row = D[k] + (int64_t)fk[k][i] * c[k];
    for (int32_t j = 0; j < c[k]; ++j) t[pos++] = row[j];
  }
}

/*
 * Y[i,:] = model(tuple_i).
 *   X      [n x c_f] row-major (may be NULL when c_f == 0)
 *   D[k]   [r_k x c_k] row-major, fk[k][i] in [0, r_k)
 *   W[j]   [w_in[j] x w_out[j]] row-major; w_in[0] = c_f + sum c_k,
 *          w_in[j] = w_out[j-1]
 *   bias[j] w_out[j] values or NULL
 *   Y      [n x w_out[n_layers-1]]
 * Returns 0, or -1 on a shape mismatch / failed allocation.
 */
int lqo_join_predict(int64_t n, int32_t c_f, const double* X, int32_t K,
                     const int32_t* c, const double* const* D,
                     const int32_t* const* fk, int32_t n_layers,
                     const int32_t* w_in, const int32_t* w_out,
                     const double* const* W, const double* const* bias,
                     double* Y, int nthreads) {
  int64_t kw = c_f;
  for (int32_t k = 0; k < K; ++k) kw += c[k];
  if (n_layers < 1 || w_in[0] != kw) return -1;
  int64_t widest = kw;
  for (int32_t j = 0; j < n_layers; ++j) {
    if (j > 0 && w_in[j] != w_out[j - 1]) return -1;
    if (w_out[j] > widest) widest = w_out[j];
  }
  const int32_t l_out = w_out[n_layers - 1];
  int failed = 0;
  nthreads = clamp_threads(nthreads);
#pragma omp parallel num_threads(nthreads)
  {
    double* a = (double*)malloc(sizeof(double) * (size_t)(widest + 1));
    double* b = (double*)malloc(sizeof(double) * (size_t)(widest + 1));
    if (!a || !b) {
#pragma omp atomic write
      failed = 1;
    } else {
#pragma omp for schedule(static)
      for (int64_t i = 0; i < n; ++i) {
        build_tuple(i, c_f, X, K, c, D, fk, a);
        for (int32_t j = 0; j < n_layers; ++j) {
          const double* Wj = W[j];
          for (int32_t o = 0; o < w_out[j]; ++o) {
            double s = 0.0;
            for (int32_t q = 0; q < w_in[j]; ++q)
              s += a[q] * Wj[(int64_t)q * w_out[j] + o];
            if (bias && bias[j]) s += bias[j][o];
            if (j < n_layers - 1 && s < 0.0) s = 0.0;
            b[o] = s;
          }
          double* tmp = a; a = b; b = tmp;
        }
        for (int32_t o = 0; o < l_out; ++o) Y[i * (int64_t)l_out + o] = a[o];
      }
    }
    free(a);
    free(b);
  }
  return failed ? -1 : 0;
}

/* T[i,:] = joined tuple of fact row i, T is [n x (c_f + sum c_k)]. */
int lqo_materialize(int64_t n, int32_t c_f, const double* X, int32_t K,
                    const int32_t* c, const double* const* D,
                    const int32_t* const* fk, double* T) {
  int64_t kw = c_f;
  for (int32_t k = 0; k < K; ++k) kw += c[k];
  for (int64_t i = 0; i < n; ++i) build_tuple(i, c_f, X, K, c, D, fk, T + i * kw);
  return 0;
}

/*
 * P = D * W[row_off : row_off + c, :],  D [r x c], W [? x l] row-major,
 * P [r x l].  row_off is where this dimension's columns sit in the tuple.
 */
int lqo_project_dims(int64_t r, int32_t c, const double* D, int32_t row_off,
                     int32_t l, const double* W, double* P) {
  for (int64_t i = 0; i < r; ++i)
    for (int32_t o = 0; o < l; ++o) {
      double s = 0.0;
      for (int32_t q = 0; q < c; ++q)
        s += D[i * c + q] * W[(int64_t)(row_off + q) * l + o];
      P[i * l + o] = s;
    }
  return 0;
}

/*
 * Z[i,:] = X[i,:] * W[0:c_f, :] + sum_k P_k[fk_k[i], :] (+ bias).
 * The right-hand side of Eq. 1 with the fact table joined by the identity.
 */
int lqo_gather_sum(int64_t n, int32_t c_f, const double* X, int32_t l,
                   const double* W, int32_t K, const double* const* P,
                   const int32_t* const* fk, const double* bias, double* Z) {
  for (int64_t i = 0; i < n; ++i)
    for (int32_t o = 0; o < l; ++o) {
      double s = 0.0;
      for (int32_t q = 0; q < c_f; ++q)
        s += X[i * (int64_t)c_f + q] * W[(int64_t)q * l + o];
      for (int32_t k = 0; k < K; ++k) s += P[k][(int64_t)fk[k][i] * l + o];
      if (bias) s += bias[o];
      Z[i * (int64_t)l + o] = s;
    }
  return 0;
}

/*
 * Filter, star-join, GROUP BY, SUM / COUNT, one tuple at a time.
 *   fk[k][i]      row of dimension k matched by fact row i; < 0 = no match
 *   dim_mask[k]   NULL or r_k bytes, 0 = the dimension row fails its predicate
 *   dim_code[k]   NULL (dimension k does not group) or r_k group codes in
 *                 [0, card[k])
 *   fact_mask     NULL or n bytes
 *   measure[m]    n int32 values
 *   sums   [n_measures x G], counts [G] (may be NULL), G = prod card[k] over
 *          grouping dimensions; both overwritten.
 * Returns 0, -1 on allocation failure, -2 if a code is outside [0, card).
 */
int lqo_groupby_sum(int64_t n, int32_t K, const int32_t* const* fk,
                    const uint8_t* const* dim_mask,
                    const int32_t* const* dim_code, const int32_t* card,
                    const uint8_t* fact_mask, int32_t n_measures,
                    const int32_t* const* measure, int64_t* sums,
                    int64_t* counts, int nthreads) {
  int64_t G = 1;
  for (int32_t k = 0; k < K; ++k)
    if (dim_code && dim_code[k]) G *= card[k];
  nthreads = clamp_threads(nthreads);
  const size_t per = (size_t)G * (size_t)(n_measures + 1);
  int64_t* priv = (int64_t*)calloc(per * (size_t)nthreads, sizeof(int64_t));
  if (!priv) return -1;
  int bad = 0;
#pragma omp parallel num_threads(nthreads)
  {
    int tid = 0, nt = 1;
#ifdef _OPENMP
    tid = omp_get_thread_num();
    nt = omp_get_num_threads();
#endif
    int64_t* s = priv + per * (size_t)tid;
    int64_t* cnt = s + (size_t)G * (size_t)n_measures;
    const int64_t lo = n * tid / nt, hi = n * (tid + 1) / nt;
    for (int64_t i = lo; i < hi; ++i) {
      if (fact_mask && !fact_mask[i]) continue;
      int keep = 1;
      int64_t g = 0;
      for (int32_t k = 0; k < K; ++k) {
        const int32_t j = fk[k][i];
        if (j < 0 || (dim_mask && dim_mask[k] && !dim_mask[k][j])) {
          keep = 0;
          break;
        }
        if (dim_code && dim_code[k]) {
          const int32_t code = dim_code[k][j];
          if (code < 0 || code >= card[k]) {
#pragma omp atomic write
            bad = 1;
            keep = 0;
            break;
          }
          g = g * card[k] + code;
        }
      }
      if (!keep) continue;
      for (int32_t m = 0; m < n_measures; ++m) s[(size_t)m * G + g] += measure[m][i];
      cnt[g] += 1;
    }
  }
  memset(sums, 0, sizeof(int64_t) * (size_t)G * (size_t)n_measures);
  if (counts) memset(counts, 0, sizeof(int64_t) * (size_t)G);
  for (int t = 0; t < nthreads; ++t) {
    const int64_t* s = priv + per * (size_t)t;
    for (size_t q = 0; q < (size_t)G * (size_t)n_measures; ++q) sums[q] += s[q];
    if (counts)
      for (int64_t g = 0; g < G; ++g) counts[g] += s[(size_t)G * n_measures + g];
  }
  free(priv);
  return bad ? -2 : 0;
}

/* ------------------------------------------------------------------------------------------
 * Decision tree in matrix form (Section 3.3.1) and its fusion with the dimensions (Eq. 2).
 *
 *   feature[q]  column of the joined table T tested by internal node q: the matrix F of step 1
 *               has its single 1 of column q in row feature[q] (F only selects columns)
 *   v[q]        threshold of node q (step 2: B = (T F > v), entries 0/1)
 *   H [p x l]   H[q][j] = +1 / -1 if node q lies on the path to leaf j and the path takes its
 *               True / False side, 0 if node q is not on that path (step 3: R = B H)
 *   h[j]        value R takes exactly when leaf j is reached.  A leaf is reached iff all its +1
 *               nodes are true and all its -1 nodes are false, i.e. R_j = number of +1 entries
 *               of column j.  (The paper words h as "the column sum of H", which cannot be meant
 *               literally for a 0/1 predicate matrix: a column with a -1 entry would then never match.)
 *   step 4      onehot[i][j] = (R[i][j] == h[j]);  leaf[i] = first j with onehot 1, -1 if none.
 * ------------------------------------------------------------------------------------------ */

/* Plain definition: materialise the tuple, then the four steps.  R (int32, [n x l]) may be NULL. */
int lqo_tree_predict(int64_t n, int32_t c_f, const double* X, int32_t K, const int32_t* c,
                     const double* const* D, const int32_t* const* fk, int32_t p, int32_t l,
                     const int32_t* feature, const double* v, const int8_t* H, int32_t* R,
                     uint8_t* onehot, int32_t* leaf) {
  int64_t kw = c_f;
  for (int32_t k = 0; k < K; ++k) kw += c[k];
  for (int32_t q = 0; q < p; ++q)
    if (feature[q] < 0 || feature[q] >= kw) return -1;
  double* t = (double*)malloc(sizeof(double) * (size_t)(kw + 1));
  int32_t* r = (int32_t*)malloc(sizeof(int32_t) * (size_t)(l + 1));
  int32_t* h = (int32_t*)malloc(sizeof(int32_t) * (size_t)(l + 1));
  if (!t || !r || !h) { free(t); free(r); free(h); return -1; }
  for (int32_t j = 0; j < l; ++j) {
    h[j] = 0;
    for (int32_t q = 0; q < p; ++q) h[j] += H[(int64_t)q * l + j] == 1;
  }
  for (int64_t i = 0; i < n; ++i) {
    build_tuple(i, c_f, X, K, c, D, fk, t);
    for (int32_t j = 0; j < l; ++j) r[j] = 0;
    for (int32_t q = 0; q < p; ++q) {
      const int b = t[feature[q]] > v[q];                 /* steps 1 and 2 */
      if (b)
        for (int32_t j = 0; j < l; ++j) r[j] += H[(int64_t)q * l + j];   /* step 3 */
    }
    int32_t first = -1;
    for (int32_t j = 0; j < l; ++j) {
      const int hit = r[j] == h[j];                       /* step 4 */
      if (R) R[i * (int64_t)l + j] = r[j];
      if (onehot) onehot[i * (int64_t)l + j] = (uint8_t)hit;
      if (hit && first < 0) first = j;
    }
    if (leaf) leaf[i] = first;
  }
  free(t); free(r); free(h);
  return 0;
}

/*
 * Pre-fused table of one dimension (the terms T_j of Eq. 2):
 *   Tk[r][j] = sum over the nodes q whose tested column belongs to this dimension of
 *              (D[r][feature[q] - col_off] > v[q]) * H[q][j].
 * Nodes testing other tables' columns contribute nothing here (they are evaluated where their
 * column lives), so that the partial tables add up to (T F > v) H.
 */
int lqo_tree_project(int64_t r, int32_t c, const double* D, int32_t col_off, int32_t p, int32_t l,
                     const int32_t* feature, const double* v, const int8_t* H, int32_t* Tk) {
  for (int64_t i = 0; i < r; ++i) {
    for (int32_t j = 0; j < l; ++j) Tk[i * l + j] = 0;
    for (int32_t q = 0; q < p; ++q) {
      const int32_t f = feature[q] - col_off;
      if (f < 0 || f >= c) continue;
      if (D[i * c + f] > v[q])
        for (int32_t j = 0; j < l; ++j) Tk[i * l + j] += H[(int64_t)q * l + j];
    }
  }
  return 0;
}

/* ------------------------------------------------------------------------------------------
 * Wider aggregate query: fact-side range predicates (selection vectors on the fact table,
 * Section 2.2), measures that are a column, the element-wise product or the difference of two
 * columns, and SUM / MIN / MAX / COUNT per group (Section 2.4).  Evaluated per tuple.
 *   pred_col[q], lo[q], hi[q]   keep row i iff lo <= pred_col[q][i] <= hi for every q
 *   op[m] : 0 = a[m][i], 1 = a[m][i] * b[m][i], 2 = a[m][i] - b[m][i]   (computed in int64)
 *   sums, mins, maxs [n_meas x G] (any may be NULL), counts [G] (may be NULL)
 *   mins / maxs of a group without rows stay at INT64_MAX / INT64_MIN.
 * Join, masks and group numbering as in lqo_groupby_sum.  Returns 0, -2 on a bad code.
 * ------------------------------------------------------------------------------------------ */
int lqo_groupby_agg(int64_t n, int32_t K, const int32_t* const* fk, const uint8_t* const* dim_mask,
                    const int32_t* const* dim_code, const int32_t* card, int32_t n_preds,
                    const int32_t* const* pred_col, const int32_t* lo, const int32_t* hi,
                    int32_t n_meas, const int32_t* op, const int32_t* const* a,
                    const int32_t* const* b, int64_t* sums, int64_t* mins, int64_t* maxs,
                    int64_t* counts) {
  int64_t G = 1;
  for (int32_t k = 0; k < K; ++k)
    if (dim_code && dim_code[k]) G *= card[k];
  for (int64_t q = 0; q < G * n_meas; ++q) {
    if (sums) sums[q] = 0;
    if (mins) mins[q] = INT64_MAX;
    if (maxs) maxs[q] = INT64_MIN;
  }
  if (counts) for (int64_t g = 0; g < G; ++g) counts[g] = 0;
  for (int64_t i = 0; i < n; ++i) {
    int keep = 1;
    for (int32_t q = 0; q < n_preds && keep; ++q)
      keep = pred_col[q][i] >= lo[q] && pred_col[q][i] <= hi[q];
    int64_t g = 0;
    for (int32_t k = 0; k < K && keep; ++k) {
      const int32_t j = fk[k][i];
      if (j < 0 || (dim_mask && dim_mask[k] && !dim_mask[k][j])) { keep = 0; break; }
      if (dim_code && dim_code[k]) {
        const int32_t code = dim_code[k][j];
        if (code < 0 || code >= card[k]) return -2;
        g = g * card[k] + code;
      }
    }
    if (!keep) continue;
    for (int32_t m = 0; m < n_meas; ++m) {
      const int64_t x = a[m][i];
      const int64_t v = op[m] == 1 ? x * (int64_t)b[m][i] : (op[m] == 2 ? x - (int64_t)b[m][i] : x);
      if (sums) sums[(int64_t)m * G + g] += v;
      if (mins && v < mins[(int64_t)m * G + g]) mins[(int64_t)m * G + g] = v;
      if (maxs && v > maxs[(int64_t)m * G + g]) maxs[(int64_t)m * G + g] = v;
    }
    if (counts) counts[g] += 1;
  }
  return 0;
}

/* ------------------------------------------------------------------------------------------
 * AVG per group from the SUM and COUNT of the same query (the aggregation functions of Section 2.4):
 *   avgs[m][g] = sums[m][g] / counts[g] in fp64 (both operands converted to double, one division),
 *   NaN for a group without rows (SQL: no such group, or NULL).
 * ------------------------------------------------------------------------------------------ */
void lqo_group_avg(int64_t n_meas, int64_t G, const int64_t* sums, const int64_t* counts, double* avgs) {
  for (int64_t m = 0; m < n_meas; ++m)
    for (int64_t g = 0; g < G; ++g)
      avgs[m * G + g] = counts[g] > 0 ? (double)sums[m * G + g] / (double)counts[g] : NAN;
}
