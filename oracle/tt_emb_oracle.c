/*
 * CPU oracle for the tensor-train (TT) embedding lookup, its gradient and one SGD step.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, plain definition that the GPU library is
 * checked against; nothing on the product path may call it.  It shares no code with the HIP
 * sources: every row does its own two matrix products, there is no deduplication, no blocking
 * and no reordering beyond what the paper's definition states.
 *
 * What is computed (paper notation in brackets):
 *   - a node id i is split mixed-radix, i1 = i/(n2*n3), i2 = (i/n3) mod n2, i3 = i mod n3
 *     [Section 4.2, the displayed formulas for i_1, i_2, i_3; Eq. "tt-embedding"];
 *   - row i of the table is G1[i1] * G2[i2] * G3[i3], evaluated left to right as two matrix
 *     products over the unfolded slices, with the partial product reshaped between them
 *     [Section 3, the paragraph after Eq. "tt-embedding": unfold each slice to
 *     R_{k-1} x (n_k R_k), multiply, reshape to (n_1..n_k) x R_k, continue];
 *   - output column j = (j1*d2 + j2)*d3 + j3 [Eq. "tt-embedding", the formula for j];
 *   - the gradient of L = sum_b <grad_b, row_b> with respect to the three cores.  The paper
 *     names this phase ("bwd") but prints no formula; it is the chain rule through the two
 *     products above, summed over all batch positions (duplicates add);
 *   - the parameter update ("upd").  The paper names no optimiser; this is plain SGD,
 *     G <- G - lr*dG, with every gradient taken from the cores as they were before the update.
 *
 * Naming: the table has N = n1*n2*n3 rows (paper: M = m1*m2*m3) of D = d1*d2*d3 floats
 * (paper: N = n1*n2*n3); the TT ranks are (1, r1, r2, 1) (paper: R_0..R_3).
 *
 * Storage of the cores (an interface shared with the library, stated in its header): each
 * slice is stored contiguously as its unfolding matrix,
 *   g1[n1][d1][r1]      G1[i1] is d1 x r1           (paper G_1(0, i1, j1, a))
 *   g2[n2][r1][d2][r2]  G2[i2] is r1 x (d2*r2)      (paper G_2(a, i2, j2, b))
 *   g3[n3][r2][d3]      G3[i3] is r2 x d3           (paper G_3(b, i3, j3, 0))
 *
 * Arithmetic: inputs are fp32 and are read exactly.  TT_ACC (default double) is the type of every
 * accumulator and intermediate; results are rounded to fp32 once, when stored.  The build with
 * -DTT_ACC=float (and OpenMP) is the same loops in fp32 and exists only to be timed.
 *
 * An id outside [0, N) yields a zero row and contributes no gradient (the library's documented
 * behaviour for such ids).
 *
 * Parity status: every function here is pinned by tests that do not use this file's formulas
 * (element-wise dense reconstruction, Kronecker special case, finite differences, Euler identity,
 * the paper's worked index example and parameter-count table).  Nothing is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef TT_ACC
#define TT_ACC double
#endif
typedef TT_ACC acc_t;

typedef struct {
  int64_t n[3]; /* n1, n2, n3 */
  int32_t d[3]; /* d1, d2, d3 */
  int32_t r[2]; /* r1, r2     */
} tto_shape;

/* Number of accumulator bytes, so that the caller can size buffers for tto_grads. */
int tto_acc_bytes(void) { return (int)sizeof(acc_t); }

int tto_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Parameter count of the three cores: sum_k R_{k-1} m_k n_k R_k  [Section 3, TT-matrix format;
 * Table "ogb-dim-tt" lists values of it]. */
int64_t tto_param_count(const tto_shape* s) {
  int64_t c1 = 1 * s->n[0] * s->d[0] * (int64_t)s->r[0];
  int64_t c2 = (int64_t)s->r[0] * s->n[1] * s->d[1] * (int64_t)s->r[1];
  int64_t c3 = (int64_t)s->r[1] * s->n[2] * s->d[2] * 1;
  return c1 + c2 + c3;
}

/* Mixed-radix split of a node id [Section 4.2]. Returns 0 when id is outside the table. */
int tto_decompose(const tto_shape* s, int64_t id, int64_t* i1, int64_t* i2, int64_t* i3) {
  int64_t N = s->n[0] * s->n[1] * s->n[2];
  if (id < 0 || id >= N) return 0;
  *i1 = id / (s->n[1] * s->n[2]);
  *i2 = (id / s->n[2]) % s->n[1];
  *i3 = id % s->n[2];
  return 1;
}

/* P = A * Bm for one id:  A = G1[i1] (d1 x r1), Bm = G2[i2] (r1 x d2*r2); P is d1 x (d2*r2),
 * which read row-major is also the reshaped (d1*d2) x r2 partial product. */
static void prefix_product(const tto_shape* s, const float* A, const float* Bm, acc_t* P) {
  const int d1 = s->d[0], r1 = s->r[0], w = s->d[1] * s->r[1];
  for (int j1 = 0; j1 < d1; ++j1)
    for (int col = 0; col < w; ++col) {
      acc_t t = 0;
      for (int a = 0; a < r1; ++a) t += (acc_t)A[j1 * r1 + a] * (acc_t)Bm[a * w + col];
      P[j1 * w + col] = t;
    }
}

/* E = P * C for one id: P is (d1*d2) x r2, C = G3[i3] (r2 x d3); E is (d1*d2) x d3 row-major,
 * i.e. the D entries of the embedding row in column order j = (j1*d2+j2)*d3+j3. */
static void row_product(const tto_shape* s, const acc_t* P, const float* C, acc_t* E) {
  const int m = s->d[0] * s->d[1], r2 = s->r[1], d3 = s->d[2];
  for (int jm = 0; jm < m; ++jm)
    for (int j3 = 0; j3 < d3; ++j3) {
      acc_t t = 0;
      for (int b = 0; b < r2; ++b) t += P[jm * r2 + b] * (acc_t)C[b * d3 + j3];
      E[jm * d3 + j3] = t;
    }
}

static const float* slice1(const tto_shape* s, const float* g1, int64_t i1) {
  return g1 + i1 * (int64_t)s->d[0] * s->r[0];
}
static const float* slice2(const tto_shape* s, const float* g2, int64_t i2) {
  return g2 + i2 * (int64_t)s->r[0] * s->d[1] * s->r[1];
}
static const float* slice3(const tto_shape* s, const float* g3, int64_t i3) {
  return g3 + i3 * (int64_t)s->r[1] * s->d[2];
}

/* Forward: out_acc[B][D] in the accumulator type (no rounding to fp32). */
void tto_forward_acc(const tto_shape* s, const float* g1, const float* g2, const float* g3,
                     const int64_t* ids, int64_t B, acc_t* out) {
  const int D = s->d[0] * s->d[1] * s->d[2];
  const int pn = s->d[0] * s->d[1] * s->r[1];
#pragma omp parallel
  {
    acc_t* P = (acc_t*)malloc(sizeof(acc_t) * (size_t)pn);
#pragma omp for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
      int64_t i1, i2, i3;
      acc_t* E = out + b * D;
      if (!tto_decompose(s, ids[b], &i1, &i2, &i3)) {
        for (int j = 0; j < D; ++j) E[j] = 0;
        continue;
      }
      prefix_product(s, slice1(s, g1, i1), slice2(s, g2, i2), P);
      row_product(s, P, slice3(s, g3, i3), E);
    }
    free(P);
  }
}

/* Forward rounded to fp32: out[B][D]. */
void tto_forward(const tto_shape* s, const float* g1, const float* g2, const float* g3,
                 const int64_t* ids, int64_t B, float* out) {
  const int D = s->d[0] * s->d[1] * s->d[2];
  const int pn = s->d[0] * s->d[1] * s->r[1];
#pragma omp parallel
  {
    acc_t* P = (acc_t*)malloc(sizeof(acc_t) * (size_t)pn);
    acc_t* E = (acc_t*)malloc(sizeof(acc_t) * (size_t)D);
#pragma omp for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
      int64_t i1, i2, i3;
      float* o = out + b * D;
      if (!tto_decompose(s, ids[b], &i1, &i2, &i3)) {
        for (int j = 0; j < D; ++j) o[j] = 0.0f;
        continue;
      }
      prefix_product(s, slice1(s, g1, i1), slice2(s, g2, i2), P);
      row_product(s, P, slice3(s, g3, i3), E);
      for (int j = 0; j < D; ++j) o[j] = (float)E[j];
    }
    free(P);
    free(E);
  }
}

/* Gradient of L = sum_b <grad_b, row_b> for one batch position, added into dg1/dg2/dg3 (full
 * core-shaped accumulator arrays).  With g = grad_b as (d1*d2) x d3:
 *   dG3[i3] += P^T g          (r2 x d3)
 *   dP       = g C^T          ((d1*d2) x r2, read as d1 x (d2*r2))
 *   dG1[i1] += dP Bm^T        (d1 x r1)
 *   dG2[i2] += A^T dP         (r1 x (d2*r2))
 */
static void row_backward(const tto_shape* s, const float* g1, const float* g2, const float* g3,
                         int64_t i1, int64_t i2, int64_t i3, const float* g, acc_t* P, acc_t* dP,
                         acc_t* dg1, acc_t* dg2, acc_t* dg3) {
  const int d1 = s->d[0], d2 = s->d[1], d3 = s->d[2], r1 = s->r[0], r2 = s->r[1];
  const int m = d1 * d2, w = d2 * r2;
  const float* A = slice1(s, g1, i1);
  const float* Bm = slice2(s, g2, i2);
  const float* C = slice3(s, g3, i3);
  acc_t* dA = dg1 + i1 * (int64_t)d1 * r1;
  acc_t* dB = dg2 + i2 * (int64_t)r1 * w;
  acc_t* dC = dg3 + i3 * (int64_t)r2 * d3;

  prefix_product(s, A, Bm, P);
  for (int b = 0; b < r2; ++b)
    for (int j3 = 0; j3 < d3; ++j3) {
      acc_t t = 0;
      for (int jm = 0; jm < m; ++jm) t += P[jm * r2 + b] * (acc_t)g[jm * d3 + j3];
      dC[b * d3 + j3] += t;
    }
  for (int jm = 0; jm < m; ++jm)
    for (int b = 0; b < r2; ++b) {
      acc_t t = 0;
      for (int j3 = 0; j3 < d3; ++j3) t += (acc_t)g[jm * d3 + j3] * (acc_t)C[b * d3 + j3];
      dP[jm * r2 + b] = t;
    }
  for (int j1 = 0; j1 < d1; ++j1)
    for (int a = 0; a < r1; ++a) {
      acc_t t = 0;
      for (int col = 0; col < w; ++col) t += dP[j1 * w + col] * (acc_t)Bm[a * w + col];
      dA[j1 * r1 + a] += t;
    }
  for (int a = 0; a < r1; ++a)
    for (int col = 0; col < w; ++col) {
      acc_t t = 0;
      for (int j1 = 0; j1 < d1; ++j1) t += (acc_t)A[j1 * r1 + a] * dP[j1 * w + col];
      dB[a * w + col] += t;
    }
}

/* Core gradients summed over the whole batch; dg1/dg2/dg3 are core-shaped arrays of the
 * accumulator type and are overwritten. */
void tto_grads(const tto_shape* s, const float* g1, const float* g2, const float* g3,
               const int64_t* ids, int64_t B, const float* grad, acc_t* dg1, acc_t* dg2,
               acc_t* dg3) {
  const int D = s->d[0] * s->d[1] * s->d[2];
  const int pn = s->d[0] * s->d[1] * s->r[1];
  const size_t c1 = (size_t)s->n[0] * s->d[0] * s->r[0];
  const size_t c2 = (size_t)s->n[1] * s->r[0] * s->d[1] * s->r[1];
  const size_t c3 = (size_t)s->n[2] * s->r[1] * s->d[2];
  memset(dg1, 0, c1 * sizeof(acc_t));
  memset(dg2, 0, c2 * sizeof(acc_t));
  memset(dg3, 0, c3 * sizeof(acc_t));
#pragma omp parallel
  {
    int nt = 1, tid = 0;
#ifdef _OPENMP
    nt = omp_get_num_threads();
    tid = omp_get_thread_num();
#endif
    /* every thread but the first sums into private buffers, added to the shared ones at the end */
    acc_t *p1 = dg1, *p2 = dg2, *p3 = dg3;
    if (tid != 0) {
      p1 = (acc_t*)calloc(c1, sizeof(acc_t));
      p2 = (acc_t*)calloc(c2, sizeof(acc_t));
      p3 = (acc_t*)calloc(c3, sizeof(acc_t));
    }
    acc_t* P = (acc_t*)malloc(sizeof(acc_t) * (size_t)pn);
    acc_t* dP = (acc_t*)malloc(sizeof(acc_t) * (size_t)pn);
    /* contiguous shares of the batch, in order, one per thread */
    int64_t lo = B * tid / nt, hi = B * (tid + 1) / nt;
    for (int64_t b = lo; b < hi; ++b) {
      int64_t i1, i2, i3;
      if (!tto_decompose(s, ids[b], &i1, &i2, &i3)) continue;
      row_backward(s, g1, g2, g3, i1, i2, i3, grad + b * D, P, dP, p1, p2, p3);
    }
    free(P);
    free(dP);
#pragma omp barrier
    if (tid != 0) {
#pragma omp critical
      {
        for (size_t k = 0; k < c1; ++k) dg1[k] += p1[k];
        for (size_t k = 0; k < c2; ++k) dg2[k] += p2[k];
        for (size_t k = 0; k < c3; ++k) dg3[k] += p3[k];
      }
      free(p1);
      free(p2);
      free(p3);
    }
  }
}

/* Backward and SGD step in place: G <- G - lr*dG, all gradients from the cores as passed in.
 * Slices that no id of the batch touches have a zero gradient, so G - lr*0 leaves them as they were. */
void tto_backward_update(const tto_shape* s, float* g1, float* g2, float* g3, const int64_t* ids,
                         int64_t B, const float* grad, float lr) {
  const size_t c1 = (size_t)s->n[0] * s->d[0] * s->r[0];
  const size_t c2 = (size_t)s->n[1] * s->r[0] * s->d[1] * s->r[1];
  const size_t c3 = (size_t)s->n[2] * s->r[1] * s->d[2];
  acc_t* dg1 = (acc_t*)malloc(c1 * sizeof(acc_t));
  acc_t* dg2 = (acc_t*)malloc(c2 * sizeof(acc_t));
  acc_t* dg3 = (acc_t*)malloc(c3 * sizeof(acc_t));
  tto_grads(s, g1, g2, g3, ids, B, grad, dg1, dg2, dg3);
  const acc_t step = (acc_t)lr;
  for (size_t k = 0; k < c1; ++k) g1[k] = (float)((acc_t)g1[k] - step * dg1[k]);
  for (size_t k = 0; k < c2; ++k) g2[k] = (float)((acc_t)g2[k] - step * dg2[k]);
  for (size_t k = 0; k < c3; ++k) g3[k] = (float)((acc_t)g3[k] - step * dg3[k]);
  free(dg1);
  free(dg2);
  free(dg3);
}
