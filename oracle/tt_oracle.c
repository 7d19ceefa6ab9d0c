/*
 * tt_oracle.c -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT PATH.
 *
 * A plain, slow CPU statement of what the Tensor-Train (TT) embedding-bag path
 * computes.  Only the test-suite, the smoke check and the benchmark's CPU
 * baseline leg may build, load or call this file; the GPU library never does,
 * and the two share no code.
 *
 * Every routine accumulates in double and rounds once to fp32 on store, with
 * loops in the order the formulas are written.  Nothing is blocked, fused or
 * reordered beyond what the cited passages state.
 *
 * Layout (fixed by the problem statement): core k is a flat fp32 array indexed
 *   G_k[r_{k-1}][i_k][j_k][r_k], row-major, with r_0 = r_3 = 1
 * (paper, Section II-B: a TT core has shape R_{k-1} x (m_k n_k) x R_k and the
 * boundary ranks are 1).  An embedding row has D = d1*d2*d3 columns and column
 *   j = (j1*d2 + j2)*d3 + j3.
 *
 * Parity pins (tests, CPU only): dense-table materialisation with a library
 * einsum, the rank-1 Kronecker closed form, the paper's printed index example,
 * torch.embedding_bag + autograd on a materialised table, exact finite
 * differences (the loss is linear in each core), and Euler's identity
 * <dG_k, G_k> = L.  No function in this file is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int64_t num_rows;
  int32_t n[3];
  int32_t d[3];
  int32_t r[4];
  const float *g1; /* [n1][d1][R1]         */
  const float *g2; /* [R1][n2][d2][R2]     */
  const float *g3; /* [R2][n3][d3]         */
} ora_table;

int ora_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Row index -> per-core TT indices (paper, Section III-B, the TT-index
 * equation): i_k = floor(i / prod_{l>k} m_l) mod m_k, i_1 most significant.
 * The paper's example M = 2x2x2 maps row 1 to (0,0,1) and row 0 to (0,0,0). */
void ora_split_index(int64_t idx, const int32_t n[3], int64_t out[3]) {
  out[2] = idx % n[2];
  out[1] = (idx / n[2]) % n[1];
  out[0] = idx / ((int64_t)n[1] * n[2]);
}

/* Left partial product of one lookup (Section III-B, "TT slice multiplication",
 * first two slices): P12[j1][j2][r2] = sum_{r1} G1[i1][j1][r1] * G2[r1][i2][j2][r2]. */
static void left_product(const ora_table *t, int64_t i1, int64_t i2, double *p12) {
  const int d1 = t->d[0], d2 = t->d[1], R1 = t->r[1], R2 = t->r[2], n2 = t->n[1];
  for (int j1 = 0; j1 < d1; ++j1)
    for (int j2 = 0; j2 < d2; ++j2)
      for (int r2 = 0; r2 < R2; ++r2) {
        double acc = 0.0;
        for (int r1 = 0; r1 < R1; ++r1) {
          double a = t->g1[((size_t)i1 * d1 + j1) * R1 + r1];
          double b = t->g2[(((size_t)r1 * n2 + i2) * d2 + j2) * R2 + r2];
          acc += a * b;
        }
        p12[((size_t)j1 * d2 + j2) * R2 + r2] = acc;
      }
}

/* One embedding row by the chain of slice products (the TT-matrix equation of
 * Section II-B evaluated left to right as Section III-B does):
 * row[j1][j2][j3] = sum_{r2} P12[j1][j2][r2] * G3[r2][i3][j3]. */
static void row_from_left(const ora_table *t, const double *p12, int64_t i3, double *row) {
  const int d1 = t->d[0], d2 = t->d[1], d3 = t->d[2], R2 = t->r[2], n3 = t->n[2];
  for (int jj = 0; jj < d1 * d2; ++jj)
    for (int j3 = 0; j3 < d3; ++j3) {
      double acc = 0.0;
      for (int r2 = 0; r2 < R2; ++r2)
        acc += p12[(size_t)jj * R2 + r2] * (double)t->g3[((size_t)r2 * n3 + i3) * d3 + j3];
      row[(size_t)jj * d3 + j3] = acc;
    }
}

/* scratch per lookup: p12 (d1 d2 R2) */
void ora_row(const ora_table *t, int64_t idx, double *row) {
  int64_t ii[3];
  ora_split_index(idx, t->n, ii);
  double *p12 = (double *)malloc(sizeof(double) * t->d[0] * t->d[1] * t->r[2]);
  left_product(t, ii[0], ii[1], p12);
  row_from_left(t, p12, ii[2], row);
  free(p12);
}

/* Forward, definition mode (Section III-B, bag equation): every lookup rebuilds
 * its row with the full chain; out[b] = sum of the rows of bag b (duplicates
 * count as often as they occur; an empty bag gives zeros). */
int ora_forward(const ora_table *t, const int64_t *indices, const int64_t *offsets,
                int64_t nnz, int64_t num_bags, float *out) {
  const int D = t->d[0] * t->d[1] * t->d[2];
  const int P = t->d[0] * t->d[1] * t->r[2];
  int bad = 0;
  (void)nnz;
#pragma omp parallel
  {
    double *p12 = (double *)malloc(sizeof(double) * P);
    double *row = (double *)malloc(sizeof(double) * D);
    double *acc = (double *)malloc(sizeof(double) * D);
#pragma omp for schedule(dynamic, 16)
    for (int64_t b = 0; b < num_bags; ++b) {
      for (int j = 0; j < D; ++j) acc[j] = 0.0;
      for (int64_t l = offsets[b]; l < offsets[b + 1]; ++l) {
        int64_t idx = indices[l];
        if (idx < 0 || idx >= t->num_rows) { bad = 1; continue; }
        int64_t ii[3];
        ora_split_index(idx, t->n, ii);
        left_product(t, ii[0], ii[1], p12);
        row_from_left(t, p12, ii[2], row);
        for (int j = 0; j < D; ++j) acc[j] += row[j];
      }
      for (int j = 0; j < D; ++j) out[(size_t)b * D + j] = (float)acc[j];
    }
    free(p12); free(row); free(acc);
  }
  return bad;
}

/* Core gradients of one lookup with output gradient g[d1][d2][d3] (Section
 * III-D, the backward equation): the gradient of slice k is
 * (product of the slices left of k)^T * g * (product of the slices right of k)^T.
 * Contributions are ADDED into core-shaped double arrays a1, a2, a3. */
static void lookup_backward(const ora_table *t, int64_t idx, const double *g,
                            double *a1, double *a2, double *a3,
                            double *p12, double *q23, double *u) {
  const int d1 = t->d[0], d2 = t->d[1], d3 = t->d[2];
  const int R1 = t->r[1], R2 = t->r[2], n2 = t->n[1], n3 = t->n[2];
  int64_t ii[3];
  ora_split_index(idx, t->n, ii);
  const int64_t i1 = ii[0], i2 = ii[1], i3 = ii[2];

  /* k = 3: left product is P12; dG3[r2][i3][j3] += sum_{j1,j2} P12[j1][j2][r2] g[j1][j2][j3] */
  left_product(t, i1, i2, p12);
  for (int r2 = 0; r2 < R2; ++r2)
    for (int j3 = 0; j3 < d3; ++j3) {
      double acc = 0.0;
      for (int jj = 0; jj < d1 * d2; ++jj)
        acc += p12[(size_t)jj * R2 + r2] * g[(size_t)jj * d3 + j3];
      a3[((size_t)r2 * n3 + i3) * d3 + j3] += acc;
    }

  /* k = 1: right product Q[r1][j2][j3] = sum_{r2} G2[r1][i2][j2][r2] G3[r2][i3][j3];
   * dG1[i1][j1][r1] += sum_{j2,j3} g[j1][j2][j3] Q[r1][j2][j3] */
  for (int r1 = 0; r1 < R1; ++r1)
    for (int j2 = 0; j2 < d2; ++j2)
      for (int j3 = 0; j3 < d3; ++j3) {
        double acc = 0.0;
        for (int r2 = 0; r2 < R2; ++r2)
          acc += (double)t->g2[(((size_t)r1 * n2 + i2) * d2 + j2) * R2 + r2] *
                 (double)t->g3[((size_t)r2 * n3 + i3) * d3 + j3];
        q23[((size_t)r1 * d2 + j2) * d3 + j3] = acc;
      }
  for (int j1 = 0; j1 < d1; ++j1)
    for (int r1 = 0; r1 < R1; ++r1) {
      double acc = 0.0;
      for (int j2 = 0; j2 < d2; ++j2)
        for (int j3 = 0; j3 < d3; ++j3)
          acc += g[((size_t)j1 * d2 + j2) * d3 + j3] * q23[((size_t)r1 * d2 + j2) * d3 + j3];
      a1[((size_t)i1 * d1 + j1) * R1 + r1] += acc;
    }

  /* k = 2: left = G1[i1] (d1 x R1), right = G3[i3] (R2 x d3):
   * u[j1][j2][r2] = sum_{j3} g[j1][j2][j3] G3[r2][i3][j3];
   * dG2[r1][i2][j2][r2] += sum_{j1} G1[i1][j1][r1] u[j1][j2][r2] */
  for (int jj = 0; jj < d1 * d2; ++jj)
    for (int r2 = 0; r2 < R2; ++r2) {
      double acc = 0.0;
      for (int j3 = 0; j3 < d3; ++j3)
        acc += g[(size_t)jj * d3 + j3] * (double)t->g3[((size_t)r2 * n3 + i3) * d3 + j3];
      u[(size_t)jj * R2 + r2] = acc;
    }
  for (int r1 = 0; r1 < R1; ++r1)
    for (int j2 = 0; j2 < d2; ++j2)
      for (int r2 = 0; r2 < R2; ++r2) {
        double acc = 0.0;
        for (int j1 = 0; j1 < d1; ++j1)
          acc += (double)t->g1[((size_t)i1 * d1 + j1) * R1 + r1] *
                 u[((size_t)j1 * d2 + j2) * R2 + r2];
        a2[(((size_t)r1 * n2 + i2) * d2 + j2) * R2 + r2] += acc;
      }
}

static size_t core_len(const ora_table *t, int k) {
  return (size_t)t->r[k] * t->n[k] * t->d[k] * t->r[k + 1];
}

/* Backward, definition mode: loop over bags, over the lookups of each bag; every
 * lookup adds its three slice gradients (gradients of repeated rows sum: this is
 * the true gradient of the bag sum).  Threads own private double accumulators
 * which are added in thread order at the end.  lookup_bag[l] is the bag that
 * holds lookup position l; the gradient comes from gd (double) or gf (float). */
static int backward_impl(const ora_table *t, const int64_t *indices, const int64_t *lookup_bag,
                         int64_t nnz,
                         const double *gd, const float *gf, int max_threads,
                         float *dg1, float *dg2, float *dg3) {
  const int D = t->d[0] * t->d[1] * t->d[2];
  const size_t L1 = core_len(t, 0), L2 = core_len(t, 1), L3 = core_len(t, 2);
  int nt = ora_max_threads();
  if (max_threads > 0 && nt > max_threads) nt = max_threads;
  double *acc = (double *)calloc((size_t)nt * (L1 + L2 + L3), sizeof(double));
  if (!acc) return -1;
  int bad = 0;
#pragma omp parallel num_threads(nt)
  {
#ifdef _OPENMP
    const int tid = omp_get_thread_num();
#else
    const int tid = 0;
#endif
    double *a1 = acc + (size_t)tid * (L1 + L2 + L3), *a2 = a1 + L1, *a3 = a2 + L2;
    double *p12 = (double *)malloc(sizeof(double) * t->d[0] * t->d[1] * t->r[2]);
    double *u = (double *)malloc(sizeof(double) * t->d[0] * t->d[1] * t->r[2]);
    double *q23 = (double *)malloc(sizeof(double) * t->r[1] * t->d[1] * t->d[2]);
    double *g = (double *)malloc(sizeof(double) * D);
#pragma omp for schedule(dynamic, 64)
    for (int64_t l = 0; l < nnz; ++l) {
      int64_t idx = indices[l];
      if (idx < 0 || idx >= t->num_rows) { bad = 1; continue; }
      const int64_t b = lookup_bag[l];
      if (gd) for (int j = 0; j < D; ++j) g[j] = gd[(size_t)b * D + j];
      else    for (int j = 0; j < D; ++j) g[j] = (double)gf[(size_t)b * D + j];
      lookup_backward(t, idx, g, a1, a2, a3, p12, q23, u);
    }
    free(p12); free(u); free(q23); free(g);
  }
  for (size_t e = 0; e < L1 + L2 + L3; ++e) {
    double s = 0.0;
    for (int k = 0; k < nt; ++k) s += acc[(size_t)k * (L1 + L2 + L3) + e];
    if (e < L1) dg1[e] = (float)s;
    else if (e < L1 + L2) dg2[e - L1] = (float)s;
    else dg3[e - L1 - L2] = (float)s;
  }
  free(acc);
  return bad;
}

int ora_backward(const ora_table *t, const int64_t *indices, const int64_t *offsets,
                 int64_t nnz, int64_t num_bags, const float *grad_out, int max_threads,
                 float *dg1, float *dg2, float *dg3) {
  int64_t *lookup_bag = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nnz > 0 ? nnz : 1));
  for (int64_t b = 0; b < num_bags; ++b)
    for (int64_t l = offsets[b]; l < offsets[b + 1]; ++l) lookup_bag[l] = b;
  int rc = backward_impl(t, indices, lookup_bag, nnz, NULL, grad_out, max_threads, dg1, dg2, dg3);
  free(lookup_bag);
  return rc;
}

/* Plain gradient descent on one core (the training algorithm's update step):
 * G <- G - lr * dG, evaluated in double and rounded once. */
void ora_sgd(float *g, const float *dg, int64_t count, float lr) {
  for (int64_t e = 0; e < count; ++e)
    g[e] = (float)((double)g[e] - (double)lr * (double)dg[e]);
}

/* ------------------------------------------------------------------------- *
 * Dedup ("fast") mode: the same sums re-associated the way Sections III-B/E
 * describe -- each DISTINCT row is rebuilt once (forward) and the output
 * gradients of all occurrences of a row are merged first, then multiplied with
 * the cores once per distinct row (backward).  Exact by linearity; used for
 * full-size parity after being checked against definition mode.
 * ------------------------------------------------------------------------- */
static int cmp_i64(const void *a, const void *b) {
  int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
  return (x > y) - (x < y);
}

/* unique sorted valid rows; returns count, writes uniq (caller: nnz entries) */
static int64_t unique_rows(const ora_table *t, const int64_t *indices, int64_t nnz, int64_t *uniq,
                           int *bad) {
  int64_t m = 0;
  for (int64_t l = 0; l < nnz; ++l) {
    if (indices[l] < 0 || indices[l] >= t->num_rows) { *bad = 1; continue; }
    uniq[m++] = indices[l];
  }
  qsort(uniq, (size_t)m, sizeof(int64_t), cmp_i64);
  int64_t u = 0;
  for (int64_t s = 0; s < m; ++s)
    if (s == 0 || uniq[s] != uniq[s - 1]) uniq[u++] = uniq[s];
  return u;
}

static int64_t find_slot(const int64_t *uniq, int64_t count, int64_t key) {
  int64_t lo = 0, hi = count - 1;
  while (lo < hi) { int64_t mid = (lo + hi) / 2; if (uniq[mid] < key) lo = mid + 1; else hi = mid; }
  return lo;
}

int ora_forward_dedup(const ora_table *t, const int64_t *indices, const int64_t *offsets,
                      int64_t nnz, int64_t num_bags, float *out) {
  const int D = t->d[0] * t->d[1] * t->d[2];
  const int P = t->d[0] * t->d[1] * t->r[2];
  int bad = 0;
  int64_t *uniq = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nnz > 0 ? nnz : 1));
  int64_t nu = unique_rows(t, indices, nnz, uniq, &bad);
  double *rows = (double *)malloc(sizeof(double) * (size_t)(nu > 0 ? nu : 1) * D);
#pragma omp parallel
  {
    double *p12 = (double *)malloc(sizeof(double) * P);
#pragma omp for schedule(dynamic, 64)
    for (int64_t s = 0; s < nu; ++s) {
      int64_t ii[3];
      ora_split_index(uniq[s], t->n, ii);
      left_product(t, ii[0], ii[1], p12);
      row_from_left(t, p12, ii[2], rows + (size_t)s * D);
    }
    free(p12);
#pragma omp for schedule(dynamic, 64)
    for (int64_t b = 0; b < num_bags; ++b) {
      double accv[1024];
      double *acc = (D <= 1024) ? accv : (double *)malloc(sizeof(double) * D);
      for (int j = 0; j < D; ++j) acc[j] = 0.0;
      for (int64_t l = offsets[b]; l < offsets[b + 1]; ++l) {
        if (indices[l] < 0 || indices[l] >= t->num_rows) continue;
        const double *row = rows + (size_t)find_slot(uniq, nu, indices[l]) * D;
        for (int j = 0; j < D; ++j) acc[j] += row[j];
      }
      for (int j = 0; j < D; ++j) out[(size_t)b * D + j] = (float)acc[j];
      if (acc != accv) free(acc);
    }
  }
  free(rows); free(uniq);
  return bad;
}

int ora_backward_dedup(const ora_table *t, const int64_t *indices, const int64_t *offsets,
                       int64_t nnz, int64_t num_bags, const float *grad_out, int max_threads,
                       float *dg1, float *dg2, float *dg3) {
  const int D = t->d[0] * t->d[1] * t->d[2];
  int bad = 0;
  int64_t *uniq = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nnz > 0 ? nnz : 1));
  int64_t nu = unique_rows(t, indices, nnz, uniq, &bad);
  /* merge the output gradients of all occurrences of each distinct row */
  double *gagg = (double *)calloc((size_t)(nu > 0 ? nu : 1) * D, sizeof(double));
  int64_t *slot_bag = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nu > 0 ? nu : 1));
  for (int64_t b = 0; b < num_bags; ++b)
    for (int64_t l = offsets[b]; l < offsets[b + 1]; ++l) {
      if (indices[l] < 0 || indices[l] >= t->num_rows) continue;
      double *dst = gagg + (size_t)find_slot(uniq, nu, indices[l]) * D;
      for (int j = 0; j < D; ++j) dst[j] += (double)grad_out[(size_t)b * D + j];
    }
  for (int64_t s = 0; s < nu; ++s) slot_bag[s] = s; /* "bag" of unique row s is its own slot */
  int rc = backward_impl(t, uniq, slot_bag, nu, gagg, NULL, max_threads, dg1, dg2, dg3);
  free(gagg); free(slot_bag); free(uniq);
  return rc < 0 ? rc : (rc | bad);
}
