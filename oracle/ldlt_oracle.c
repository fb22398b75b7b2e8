/*
 * CPU oracle for log|det A| and sign(det A) of a symmetric matrix.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the GPU
 * library is checked against.  It shares no code with the HIP path, is never
 * called by it, and must only be used from tests, the smoke check and the
 * benchmark's CPU-baseline leg.
 *
 * What it computes.  The paper's method (Sec. 2.2, Eq. 1 and the paragraph after
 * it; App. D) reaches, up to rounding, the exact log-determinant: the sum of the
 * log-determinants of the diagonal factors met while the Schur complement is
 * reduced block by block.  For the symmetric case the factorisation is
 * A = L D L^T with unit lower-triangular L and diagonal D (Sec. 2.2, last two
 * paragraphs; App. D first paragraph: the factorisation also yields the
 * determinants of all leading principal sub-matrices), so
 *
 *      log|det A| = sum_j log|d_j| ,     sign det A = prod_j sgn d_j .
 *
 * The oracle is that definition written out, unblocked, without pivoting, in
 * `long double` (x87 80-bit, 64-bit significand):
 *
 *      d_j  = a_jj - sum_{k<j} l_jk^2 d_k
 *      l_ij = (a_ij - sum_{k<j} l_ik l_jk d_k) / d_j        (i > j)
 *
 * Only the lower triangle of the row-major input is read.  The input bits
 * (double or float) are converted exactly to long double.
 *
 * The only parallelism is an OpenMP `parallel for` over the rows i of one
 * pivot column j; the summation order inside every dot product is k = 0..j-1.
 *
 * Also here: a brute-force Leibniz determinant (sum over all permutations),
 * used to pin the factorisation on tiny matrices; and the same plain reference
 * for the positive-definite form of the method (the paper's algorithm for
 * symmetric positive-definite matrices; App. D: M = L L^T with lower-triangular
 * L gives logdet(M[:k,:k]) = 2 sum_{i<=k} log L_ii), unblocked Cholesky in
 * long double:
 *
 *      l_jj = sqrt(a_jj - sum_{k<j} l_jk^2)
 *      l_ij = (a_ij - sum_{k<j} l_ik l_jk) / l_jj           (i > j)
 *
 * And the symmetric case with a permutation, P A P^T = L D L^T (Sec. 2.2: the
 * symmetric form handles permutations and the diagonal scaling; pivoting is
 * confined to a block, there is none between blocks; the software section lists
 * `perm` among the outputs): elimination on the whole symmetric matrix, where at
 * step j the pivot is the entry of largest magnitude on the diagonal of the
 * current Schur complement among the indices of j's group of `group` consecutive
 * indices (on ties the one that came first in the input), brought to position j by
 * swapping rows and columns.  See ldlt_pivoted_core.
 *
 * And the generic case (Sec. 2.2, Eq. 1 and Alg. 1: M = P L U, the determinant is the
 * product of the pivots times the sign of the permutation; pivoting inside a block, none
 * between blocks): Gaussian elimination on the full matrix with the pivot of column j
 * taken among the rows of j's group of `group` consecutive indices.  See lu_core.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

typedef long double xreal;

/* Row i of the strictly-lower factor is stored packed: i entries. */
static inline size_t row_off(size_t i) { return i * (i - 1) / 2; }

/*
 * Core recurrence.  `get(ctx, i, j)` returns a_ij (i >= j) as long double.
 * Outputs (any may be NULL):
 *   d_out[n]       pivots d_j rounded to double
 *   cum_out[n]     running sums  sum_{j<=k} log|d_j|  (log-determinants of the
 *                  leading principal sub-matrices), rounded to double
 *   l_out[n*n]     row-major unit lower factor L (upper part zero), double
 * Returns 0 on success, 1 if an exact zero pivot was met (then *sign = 0,
 * *logabsdet = -inf, *bad = its index), 2 on allocation failure.
 */
typedef xreal (*getter)(const void *ctx, size_t i, size_t j, size_t lda);

static xreal get_f64(const void *a, size_t i, size_t j, size_t lda) {
  return (xreal)((const double *)a)[i * lda + j];
}
static xreal get_f32(const void *a, size_t i, size_t j, size_t lda) {
  return (xreal)((const float *)a)[i * lda + j];
}

static int ldlt_core(const void *a, size_t n, size_t lda, getter get,
                     double *logabsdet, int *sign, int64_t *bad,
                     int64_t *negative, double *d_out, double *cum_out,
                     double *l_out) {
  *logabsdet = 0.0;
  *sign = 1;
  if (bad) *bad = -1;
  if (negative) *negative = 0;
  if (n == 0) return 0;

  size_t nl = n * (n - 1) / 2;
  xreal *l = (xreal *)malloc((nl ? nl : 1) * sizeof(xreal));
  xreal *d = (xreal *)malloc(n * sizeof(xreal));
  xreal *v = (xreal *)malloc(n * sizeof(xreal)); /* v_k = l_jk d_k */
  if (!l || !d || !v) {
    free(l); free(d); free(v);
    return 2;
  }

  int status = 0;
  xreal acc_log = 0.0L;
  int sg = 1;
  int64_t neg = 0;

  for (size_t j = 0; j < n; ++j) {
    const xreal *lj = l + (j ? row_off(j) : 0);
    xreal s = get(a, j, j, lda);
    for (size_t k = 0; k < j; ++k) {
      v[k] = lj[k] * d[k];
      s -= lj[k] * v[k];
    }
    d[j] = s;
    if (s == 0.0L) {
      status = 1;
      if (bad) *bad = (int64_t)j;
      break;
    }
    if (s < 0.0L) { sg = -sg; ++neg; }
    acc_log += logl(fabsl(s));
    if (cum_out) cum_out[j] = (double)acc_log;

    long i;
#pragma omp parallel for schedule(static)
    for (i = (long)j + 1; i < (long)n; ++i) {
      xreal *li = l + row_off((size_t)i);
      xreal t = get(a, (size_t)i, j, lda);
      for (size_t k = 0; k < j; ++k) t -= li[k] * v[k];
      li[j] = t / s;
    }
  }

  if (status == 0) {
    *logabsdet = (double)acc_log;
    *sign = sg;
  } else {
    *logabsdet = -INFINITY;
    *sign = 0;
  }
  if (negative) *negative = neg;
  if (d_out)
    for (size_t j = 0; j < n; ++j) d_out[j] = (double)d[j];
  if (l_out && status == 0) {
    memset(l_out, 0, n * n * sizeof(double));
    for (size_t i = 0; i < n; ++i) {
      for (size_t k = 0; k < i; ++k) l_out[i * n + k] = (double)l[row_off(i) + k];
      l_out[i * n + i] = 1.0;
    }
  }
  free(l); free(d); free(v);
  return status;
}

int oracle_ldlt_f64(const double *a, int64_t n, int64_t lda, double *logabsdet,
                    int *sign, int64_t *bad, int64_t *negative, double *d_out,
                    double *cum_out, double *l_out) {
  return ldlt_core(a, (size_t)n, (size_t)lda, get_f64, logabsdet, sign, bad,
                   negative, d_out, cum_out, l_out);
}

int oracle_ldlt_f32(const float *a, int64_t n, int64_t lda, double *logabsdet,
                    int *sign, int64_t *bad, int64_t *negative, double *d_out,
                    double *cum_out, double *l_out) {
  return ldlt_core(a, (size_t)n, (size_t)lda, get_f32, logabsdet, sign, bad,
                   negative, d_out, cum_out, l_out);
}

/*
 * LDL^T with diagonal pivoting inside groups of `group` consecutive indices.
 *
 * Works on a full long-double copy S of the symmetric matrix (built from the lower
 * triangle of the input).  Step j, with hi = end of j's group:
 *     p      = argmax_{j <= k < hi} |S_kk|   (on ties the candidate with the smallest
 *              index in the input)                                   if choose != 0,
 *              j                                                     otherwise;
 *     slack_j = |S_pp| / max_{j <= k < hi} |S_kk|   (1 when the maximum was chosen);
 *     swap rows and columns j <-> p of S (rows of the finished part of L with them),
 *     d_j = S_jj,  l_ij = S_ij / d_j,  S_ik -= l_ij d_j l_kj   for i, k > j.
 * perm_out[j] = original index of the row/column that ended at position j, so that
 * A[perm][:, perm] = L D L^T.  With choose == 0 nothing is swapped: the plain
 * factorisation in right-looking order, slack_j then tells how far each pivot was
 * from the one the rule would have chosen (the caller permutes the input first to
 * check somebody else's permutation).
 * Outputs (any may be NULL): perm_out[n], slack_out[n], d_out[n], l_out[n*n] (unit
 * lower L, row-major).  Returns 0, 1 on an exact zero pivot (then *bad = j, sign 0,
 * logabsdet -inf), 2 on allocation failure or group < 1.
 */
static int ldlt_pivoted_core(const void *a, size_t n, size_t lda, getter get, size_t group,
                             int choose, double *logabsdet, int *sign, int64_t *bad,
                             int64_t *negative, int64_t *perm_out, double *slack_out,
                             double *d_out, double *l_out) {
  *logabsdet = 0.0;
  *sign = 1;
  if (bad) *bad = -1;
  if (negative) *negative = 0;
  if (group < 1) return 2;
  if (n == 0) return 0;
  xreal *S = (xreal *)malloc(n * n * sizeof(xreal));
  size_t *perm = (size_t *)malloc(n * sizeof(size_t));
  if (!S || !perm) { free(S); free(perm); return 2; }
  for (size_t i = 0; i < n; ++i) {
    perm[i] = i;
    for (size_t k = 0; k <= i; ++k) S[i * n + k] = S[k * n + i] = get(a, i, k, lda);
  }
  int status = 0, sg = 1;
  int64_t neg = 0;
  xreal acc_log = 0.0L;
  for (size_t j = 0; j < n; ++j) {
    size_t hi = (j / group + 1) * group;
    if (hi > n) hi = n;
    /* among equal magnitudes the candidate that came first in the input: a rule that
       does not depend on where the swaps of earlier steps have put the candidates */
    size_t best = j;
    for (size_t k = j + 1; k < hi; ++k) {
      const xreal vk = fabsl(S[k * n + k]), vb = fabsl(S[best * n + best]);
      if (vk > vb || (vk == vb && perm[k] < perm[best])) best = k;
    }
    const size_t p = choose ? best : j;
    const xreal top = fabsl(S[best * n + best]);
    if (slack_out) slack_out[j] = top == 0.0L ? 1.0 : (double)(fabsl(S[p * n + p]) / top);
    if (p != j) {
      for (size_t k = 0; k < n; ++k) { xreal t = S[j * n + k]; S[j * n + k] = S[p * n + k]; S[p * n + k] = t; }
      for (size_t k = 0; k < n; ++k) { xreal t = S[k * n + j]; S[k * n + j] = S[k * n + p]; S[k * n + p] = t; }
      size_t t = perm[j]; perm[j] = perm[p]; perm[p] = t;
    }
    const xreal d = S[j * n + j];
    if (d == 0.0L) {
      status = 1;
      if (bad) *bad = (int64_t)j;
      break;
    }
    if (d < 0.0L) { sg = -sg; ++neg; }
    acc_log += logl(fabsl(d));
    /* row j right of the diagonal keeps the un-normalised column, w_k = l_kj d_j; every
       updated entry is written to both triangles, so S stays exactly symmetric */
    long i;
#pragma omp parallel for schedule(static)
    for (i = (long)j + 1; i < (long)n; ++i) {
      const size_t r = (size_t)i;
      const xreal l = S[r * n + j] / d;
      for (size_t k = j + 1; k <= r; ++k) {
        const xreal v = S[r * n + k] - l * S[j * n + k];
        S[r * n + k] = v;
        S[k * n + r] = v;
      }
      S[r * n + j] = l;
    }
  }
  if (status == 0) { *logabsdet = (double)acc_log; *sign = sg; }
  else { *logabsdet = -INFINITY; *sign = 0; }
  if (negative) *negative = neg;
  if (perm_out) for (size_t j = 0; j < n; ++j) perm_out[j] = (int64_t)perm[j];
  if (d_out) for (size_t j = 0; j < n; ++j) d_out[j] = (double)S[j * n + j];
  if (l_out && status == 0) {
    memset(l_out, 0, n * n * sizeof(double));
    for (size_t i = 0; i < n; ++i) {
      for (size_t k = 0; k < i; ++k) l_out[i * n + k] = (double)S[i * n + k];
      l_out[i * n + i] = 1.0;
    }
  }
  free(S); free(perm);
  return status;
}

int oracle_ldlt_pivoted_f64(const double *a, int64_t n, int64_t lda, int64_t group, int choose,
                            double *logabsdet, int *sign, int64_t *bad, int64_t *negative,
                            int64_t *perm_out, double *slack_out, double *d_out, double *l_out) {
  return ldlt_pivoted_core(a, (size_t)n, (size_t)lda, get_f64, group < 1 ? 0 : (size_t)group, choose,
                           logabsdet, sign, bad, negative, perm_out, slack_out, d_out, l_out);
}

int oracle_ldlt_pivoted_f32(const float *a, int64_t n, int64_t lda, int64_t group, int choose,
                            double *logabsdet, int *sign, int64_t *bad, int64_t *negative,
                            int64_t *perm_out, double *slack_out, double *d_out, double *l_out) {
  return ldlt_pivoted_core(a, (size_t)n, (size_t)lda, get_f32, group < 1 ? 0 : (size_t)group, choose,
                           logabsdet, sign, bad, negative, perm_out, slack_out, d_out, l_out);
}

/*
 * LU with partial (row) pivoting inside groups of `group` consecutive rows.
 *
 * Works on a full long-double copy S of the matrix (all n x n entries are read).  Step j,
 * with hi = end of j's group:
 *     p = argmax_{j <= r < hi} |S_rj|   (on ties the row that came first in the input);
 *     swap rows j <-> p of S (the finished part of L with them); sign flips if p != j;
 *     d_j = S_jj,  l_rj = S_rj / d_j,  S_rc -= l_rj S_jc   for r, c > j.
 * perm_out[j] = original index of the row that ended at position j: A[perm, :] = L U with
 * unit lower L and upper U, U_jj = d_j.  Outputs (any may be NULL): perm_out[n], d_out[n],
 * lu_out[n*n] (row-major: L strictly below the diagonal, U on and above it).
 * *sign = sign of the permutation times the signs of the pivots.  Returns 0, 1 on an exact
 * zero pivot (every candidate of the column is zero; then *bad = j, sign 0, logabsdet
 * -inf), 2 on allocation failure or group < 1.
 */
static xreal getfull_f64(const void *a, size_t i, size_t j, size_t lda) {
  return (xreal)((const double *)a)[i * lda + j];
}
static xreal getfull_f32(const void *a, size_t i, size_t j, size_t lda) {
  return (xreal)((const float *)a)[i * lda + j];
}
static int lu_core(const void *a, size_t n, size_t lda, getter get, size_t group, double *logabsdet,
                   int *sign, int64_t *bad, int64_t *negative, int64_t *perm_out, double *d_out,
                   double *lu_out) {
  *logabsdet = 0.0;
  *sign = 1;
  if (bad) *bad = -1;
  if (negative) *negative = 0;
  if (group < 1) return 2;
  if (n == 0) return 0;
  xreal *S = (xreal *)malloc(n * n * sizeof(xreal));
  size_t *perm = (size_t *)malloc(n * sizeof(size_t));
  if (!S || !perm) { free(S); free(perm); return 2; }
  for (size_t i = 0; i < n; ++i) {
    perm[i] = i;
    for (size_t k = 0; k < n; ++k) S[i * n + k] = get(a, i, k, lda);
  }
  int status = 0, sg = 1;
  int64_t neg = 0;
  xreal acc_log = 0.0L;
  for (size_t j = 0; j < n; ++j) {
    size_t hi = (j / group + 1) * group;
    if (hi > n) hi = n;
    size_t p = j;
    for (size_t r = j + 1; r < hi; ++r) {
      const xreal vr = fabsl(S[r * n + j]), vp = fabsl(S[p * n + j]);
      if (vr > vp || (vr == vp && perm[r] < perm[p])) p = r;
    }
    if (p != j) {
      for (size_t k = 0; k < n; ++k) { xreal t = S[j * n + k]; S[j * n + k] = S[p * n + k]; S[p * n + k] = t; }
      size_t t = perm[j]; perm[j] = perm[p]; perm[p] = t;
      sg = -sg;
    }
    const xreal d = S[j * n + j];
    if (d == 0.0L) {
      status = 1;
      if (bad) *bad = (int64_t)j;
      break;
    }
    if (d < 0.0L) { sg = -sg; ++neg; }
    acc_log += logl(fabsl(d));
    long i;
#pragma omp parallel for schedule(static)
    for (i = (long)j + 1; i < (long)n; ++i) {
      const size_t r = (size_t)i;
      const xreal l = S[r * n + j] / d;
      for (size_t c = j + 1; c < n; ++c) S[r * n + c] -= l * S[j * n + c];
      S[r * n + j] = l;
    }
  }
  if (status == 0) { *logabsdet = (double)acc_log; *sign = sg; }
  else { *logabsdet = -INFINITY; *sign = 0; }
  if (negative) *negative = neg;
  if (perm_out) for (size_t j = 0; j < n; ++j) perm_out[j] = (int64_t)perm[j];
  if (d_out) for (size_t j = 0; j < n; ++j) d_out[j] = (double)S[j * n + j];
  if (lu_out && status == 0) for (size_t e = 0; e < n * n; ++e) lu_out[e] = (double)S[e];
  free(S); free(perm);
  return status;
}

int oracle_lu_f64(const double *a, int64_t n, int64_t lda, int64_t group, double *logabsdet, int *sign,
                  int64_t *bad, int64_t *negative, int64_t *perm_out, double *d_out, double *lu_out) {
  return lu_core(a, (size_t)n, (size_t)lda, getfull_f64, group < 1 ? 0 : (size_t)group, logabsdet, sign,
                 bad, negative, perm_out, d_out, lu_out);
}

int oracle_lu_f32(const float *a, int64_t n, int64_t lda, int64_t group, double *logabsdet, int *sign,
                  int64_t *bad, int64_t *negative, int64_t *perm_out, double *d_out, double *lu_out) {
  return lu_core(a, (size_t)n, (size_t)lda, getfull_f32, group < 1 ? 0 : (size_t)group, logabsdet, sign,
                 bad, negative, perm_out, d_out, lu_out);
}

/*
 * Cholesky recurrence.  Outputs (any may be NULL): diag_out[n] = l_jj,
 * cum_out[n] = 2 sum_{j<=k} log l_jj, l_out[n*n] = row-major L (upper part zero).
 * Returns 0 on success, 3 if a pivot a_jj - sum l_jk^2 is not positive (then
 * *bad = its index and *logdet = NaN), 2 on allocation failure.
 */
static int chol_core(const void *a, size_t n, size_t lda, getter get, double *logdet,
                     int64_t *bad, double *diag_out, double *cum_out, double *l_out) {
  *logdet = 0.0;
  if (bad) *bad = -1;
  if (n == 0) return 0;
  xreal *l = (xreal *)malloc(n * (n + 1) / 2 * sizeof(xreal)); /* row i: i + 1 entries */
  if (!l) return 2;
  int status = 0;
  xreal acc_log = 0.0L;
  for (size_t j = 0; j < n; ++j) {
    xreal *lj = l + j * (j + 1) / 2;
    xreal s = get(a, j, j, lda);
    for (size_t k = 0; k < j; ++k) s -= lj[k] * lj[k];
    if (!(s > 0.0L)) {
      status = 3;
      if (bad) *bad = (int64_t)j;
      break;
    }
    const xreal ljj = sqrtl(s);
    lj[j] = ljj;
    acc_log += 2.0L * logl(ljj);
    if (cum_out) cum_out[j] = (double)acc_log;
    if (diag_out) diag_out[j] = (double)ljj;
    long i;
#pragma omp parallel for schedule(static)
    for (i = (long)j + 1; i < (long)n; ++i) {
      xreal *li = l + (size_t)i * ((size_t)i + 1) / 2;
      xreal t = get(a, (size_t)i, j, lda);
      for (size_t k = 0; k < j; ++k) t -= li[k] * lj[k];
      li[j] = t / ljj;
    }
  }
  *logdet = status == 0 ? (double)acc_log : NAN;
  if (l_out && status == 0) {
    memset(l_out, 0, n * n * sizeof(double));
    for (size_t i = 0; i < n; ++i)
      for (size_t k = 0; k <= i; ++k) l_out[i * n + k] = (double)l[i * (i + 1) / 2 + k];
  }
  free(l);
  return status;
}

int oracle_cholesky_f64(const double *a, int64_t n, int64_t lda, double *logdet, int64_t *bad,
                        double *diag_out, double *cum_out, double *l_out) {
  return chol_core(a, (size_t)n, (size_t)lda, get_f64, logdet, bad, diag_out, cum_out, l_out);
}

int oracle_cholesky_f32(const float *a, int64_t n, int64_t lda, double *logdet, int64_t *bad,
                        double *diag_out, double *cum_out, double *l_out) {
  return chol_core(a, (size_t)n, (size_t)lda, get_f32, logdet, bad, diag_out, cum_out, l_out);
}

/*
 * Leibniz formula: det A = sum over permutations p of sgn(p) prod_i a_{i,p(i)}.
 * Reads the FULL n x n row-major matrix (so it also serves non-symmetric
 * checks).  n <= 10.  Returns log|det| and sign; det itself via *det_out
 * (long double rounded to double) when not NULL.
 */
static void leibniz_rec(const double *a, int n, int row, unsigned used,
                        xreal prod, int inv_parity, xreal *acc) {
  if (row == n) {
    *acc += inv_parity ? -prod : prod;
    return;
  }
  for (int c = 0; c < n; ++c) {
    if (used & (1u << c)) continue;
    /* inversions added by putting column c in this row: columns > c already used */
    int inv = 0;
    for (int c2 = c + 1; c2 < n; ++c2)
      if (used & (1u << c2)) ++inv;
    leibniz_rec(a, n, row + 1, used | (1u << c),
                prod * (xreal)a[row * n + c], inv_parity ^ (inv & 1), acc);
  }
}

int oracle_leibniz_f64(const double *a, int n, double *logabsdet, int *sign,
                       double *det_out) {
  if (n < 0 || n > 10) return 2;
  xreal acc = 0.0L;
  if (n == 0) acc = 1.0L;
  else leibniz_rec(a, n, 0, 0u, 1.0L, 0, &acc);
  if (det_out) *det_out = (double)acc;
  if (acc == 0.0L) { *logabsdet = -INFINITY; *sign = 0; }
  else { *logabsdet = (double)logl(fabsl(acc)); *sign = acc > 0 ? 1 : -1; }
  return 0;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
