/*
 * CPU oracle for the sparse GNN hot path: SpMM, cached-transpose backward, SDDMM, FusedMM.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the GPU library is
 * checked against.  It shares no code with the GPU library; only tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it.  Every floating-point result is accumulated
 * and returned in fp64.
 *
 * What each function follows (iSpLib paper, arXiv 2403.14853):
 *   - SpMM, sum reduction, sparse operand in CSR, dense operand a 2-d row-major matrix:
 *     abstract, Section 1 (the two sparse operations), Section 3.4 (sum is the standard
 *     reduction), Section 3.5 (CSR sparse operand + dense 2-d operand).  The paper states
 *     (Section 5) that its SpMM returns the same results as PyTorch's, so the oracle is the
 *     textbook definition written as one loop nest.
 *   - Backward of SpMM through a transpose computed once and reused across epochs:
 *     Section 3.3 (cache-enabled backpropagation).  The paper does not say which expression
 *     is cached; the reading taken here is the CSR transpose.  The transpose is a stable
 *     counting sort by column, which makes it unique.
 *   - SDDMM (sampled dense-dense product, one dot product per stored entry): Section 1.
 *   - FusedMM (SDDMM -> edge function -> SpMM without materialising the edge matrix):
 *     Section 1(a).  The paper gives no formula; the form taken is s_ij = f(<x_i, x_j>),
 *     y_i = sum_j a_ij s_ij x_j with f the sigmoid (the benchmark's instance), the identity or
 *     the constant one.  Its backward is derived by the chain rule (the paper is silent) and
 *     pinned by finite differences in the tests.
 *
 * Parity pins (tests/test_oracle_*.py): dense brute force, scipy, closed forms, adjoint
 * identities, finite differences; the error-scale outputs (mag) are each recomputed in dense
 * fp64 from their formulas.  No function or output here is unpinned.
 *
 * Conventions: indptr int64[n_rows+1], indices int32[nnz], values float[nnz] or NULL (= all
 * ones); dense matrices fp32 row-major with leading dimension ld (elements).  Rows may hold
 * unsorted columns and duplicates; duplicates are separate stored entries.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC isp_oracle.c -o libisp_oracle.so -lm
 * The row loops carry an OpenMP parallel-for (rows are independent); per-row arithmetic and
 * order are unchanged by it.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int isp_oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void isp_oracle_set_threads(int t) {
#ifdef _OPENMP
  if (t > 0) omp_set_num_threads(t);
#else
  (void)t;
#endif
}

/* Transpose by stable counting sort on the column index (Section 3.3 reading).
 * Entry p of A (row i, column c) lands at position q in A^T's row c; entries of one column keep
 * their source order.  t_indices[q] = i, perm[q] = p, t_values[q] = values[p].
 * values / t_values may be NULL.  Returns 0, or -1 on an out-of-range column. */
int isp_oracle_transpose(int64_t n_rows, int64_t n_cols, const int64_t* indptr, const int32_t* indices,
                         const float* values, int64_t* t_indptr, int32_t* t_indices, int32_t* perm,
                         float* t_values) {
  const int64_t nnz = indptr[n_rows];
  int64_t* cursor = (int64_t*)calloc((size_t)n_cols + 1, sizeof(int64_t));
  if (!cursor) return -2;
  for (int64_t p = 0; p < nnz; ++p) {
    if (indices[p] < 0 || indices[p] >= n_cols) { free(cursor); return -1; }
    cursor[indices[p]]++;
  }
  int64_t run = 0;
  for (int64_t c = 0; c < n_cols; ++c) {
    t_indptr[c] = run;
    run += cursor[c];
    cursor[c] = t_indptr[c];
  }
  t_indptr[n_cols] = run;
  for (int64_t i = 0; i < n_rows; ++i) {
    for (int64_t p = indptr[i]; p < indptr[i + 1]; ++p) {
      const int64_t q = cursor[indices[p]]++;
      t_indices[q] = (int32_t)i;
      perm[q] = (int32_t)p;
      if (t_values) t_values[q] = values ? values[p] : 1.0f;
    }
  }
  free(cursor);
  return 0;
}

/* SpMM, sum reduction: Y[i,k] = sum_{p in row i} a_p * X[col_p, k], stored order, fp64.
 * mag[i,k] = sum_p |a_p * X[col_p,k]| (the scale the parity tolerance is relative to); may be NULL. */
void isp_oracle_spmm(int64_t n_rows, const int64_t* indptr, const int32_t* indices, const float* values,
                     const float* X, int64_t ldx, int32_t d, double* Y, double* mag) {
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t i = 0; i < n_rows; ++i) {
    double* y = Y + i * (int64_t)d;
    double* m = mag ? mag + i * (int64_t)d : NULL;
    for (int32_t k = 0; k < d; ++k) y[k] = 0.0;
    if (m) for (int32_t k = 0; k < d; ++k) m[k] = 0.0;
    for (int64_t p = indptr[i]; p < indptr[i + 1]; ++p) {
      const double a = values ? (double)values[p] : 1.0;
      const float* x = X + (int64_t)indices[p] * ldx;
      for (int32_t k = 0; k < d; ++k) {
        const double t = a * (double)x[k];
        y[k] += t;
        if (m) m[k] += fabs(t);
      }
    }
  }
}

/* Backward of SpMM in scatter form, dX[col_p,:] += a_p * dY[i,:], without any transpose:
 * an independent second route to A^T dY.  dX is n_cols x d, zeroed here.  Sequential. */
void isp_oracle_spmm_scatter(int64_t n_rows, int64_t n_cols, const int64_t* indptr, const int32_t* indices,
                             const float* values, const float* dY, int64_t ldy, int32_t d, double* dX) {
  memset(dX, 0, (size_t)n_cols * (size_t)d * sizeof(double));
  for (int64_t i = 0; i < n_rows; ++i) {
    const float* g = dY + i * ldy;
    for (int64_t p = indptr[i]; p < indptr[i + 1]; ++p) {
      const double a = values ? (double)values[p] : 1.0;
      double* o = dX + (int64_t)indices[p] * d;
      for (int32_t k = 0; k < d; ++k) o[k] += a * (double)g[k];
    }
  }
}

/* SDDMM: out[p] = <U[i,:], V[col_p,:]> for every stored entry p of row i, in A's order;
 * multiplied by a_p when scale_by_a != 0.  mag[p] = sum_k |U[i,k] V[col_p,k]| (times |a_p|). */
void isp_oracle_sddmm(int64_t n_rows, const int64_t* indptr, const int32_t* indices, const float* values,
                      const float* U, int64_t ldu, const float* V, int64_t ldv, int32_t d, int scale_by_a,
                      double* out, double* mag) {
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t i = 0; i < n_rows; ++i) {
    const float* u = U + i * ldu;
    for (int64_t p = indptr[i]; p < indptr[i + 1]; ++p) {
      const float* v = V + (int64_t)indices[p] * ldv;
      double acc = 0.0, am = 0.0;
      for (int32_t k = 0; k < d; ++k) {
        const double t = (double)u[k] * (double)v[k];
        acc += t;
        am += fabs(t);
      }
      const double a = (scale_by_a && values) ? (double)values[p] : 1.0;
      out[p] = a * acc;
      if (mag) mag[p] = fabs(a) * am;
    }
  }
}

/* Edge functions of FusedMM: the score s = f(z) of an entry from z = <x_i, x_j>, its derivative, and
 * bounds L1 >= |f'|, L2 >= |f''| used only for the error-scale output.
 *   op 0: sigmoid, f = 1/(1+exp(-z));   op 1: identity, f = z;   op 2: constant one (plain aggregation). */
static double edge_f(int op, double z) { return op == 0 ? 1.0 / (1.0 + exp(-z)) : (op == 1 ? z : 1.0); }
static double edge_df(int op, double z) {
  if (op == 0) { const double s = 1.0 / (1.0 + exp(-z)); return s * (1.0 - s); }
  return op == 1 ? 1.0 : 0.0;
}
static double edge_l1(int op) { return op == 0 ? 0.25 : (op == 1 ? 1.0 : 0.0); }
static double edge_l2(int op) { return op == 0 ? 0.1 : 0.0; }

/* FusedMM forward (square A):
 *   z_p = <x_i, x_j>, s_p = f(z_p), Y[i,:] = sum_{p in row i} a_p s_p x_j, j = col_p.
 * mag[i,k] = sum_p |a_p| (|s_p| + L1 * sum_k' |x_ik' x_jk'|) |x_jk|: first-order error scale of the
 * fp32 evaluation (L1 bounds the edge function's derivative: 1/4 for the sigmoid). */
void isp_oracle_fusedmm(int64_t n_rows, const int64_t* indptr, const int32_t* indices, const float* values,
                        const float* X, int64_t ldx, int32_t d, int op, double* Y, double* mag) {
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t i = 0; i < n_rows; ++i) {
    const float* xi = X + i * ldx;
    double* y = Y + i * (int64_t)d;
    double* m = mag ? mag + i * (int64_t)d : NULL;
    for (int32_t k = 0; k < d; ++k) y[k] = 0.0;
    if (m) for (int32_t k = 0; k < d; ++k) m[k] = 0.0;
    for (int64_t p = indptr[i]; p < indptr[i + 1]; ++p) {
      const float* xj = X + (int64_t)indices[p] * ldx;
      double z = 0.0, za = 0.0;
      for (int32_t k = 0; k < d; ++k) {
        const double t = (double)xi[k] * (double)xj[k];
        z += t;
        za += fabs(t);
      }
      const double s = edge_f(op, z);
      const double a = values ? (double)values[p] : 1.0;
      for (int32_t k = 0; k < d; ++k) {
        y[k] += a * s * (double)xj[k];
        if (m) m[k] += fabs(a) * (fabs(s) + edge_l1(op) * za) * fabs((double)xj[k]);
      }
    }
  }
}

/* FusedMM backward, chain rule on the forward above.  With g = dY, for entry p = (i, j):
 *   ds_p = a_p <g_i, x_j>,  dz_p = ds_p f'(z_p),
 *   dX[i,:] += dz_p x_j                      (x_i enters only through z_p)
 *   dX[j,:] += a_p s_p g_i + dz_p x_i        (x_j enters directly and through z_p)
 * Scatter form, sequential.  dX is n x d, zeroed here.
 * mag[r,k] accumulates first-order error scales of the same terms: with za = sum_k |x_ik x_jk| and
 * ga = sum_k |g_ik x_jk|, |dz| is replaced by |a_p| ga (|f'| + L2 za) and s by |s| + L1 za. */
void isp_oracle_fusedmm_backward(int64_t n, const int64_t* indptr, const int32_t* indices, const float* values,
                                 const float* X, int64_t ldx, const float* dY, int64_t ldg, int32_t d, int op,
                                 double* dX, double* mag) {
  memset(dX, 0, (size_t)n * (size_t)d * sizeof(double));
  if (mag) memset(mag, 0, (size_t)n * (size_t)d * sizeof(double));
  for (int64_t i = 0; i < n; ++i) {
    const float* xi = X + i * ldx;
    const float* gi = dY + i * ldg;
    for (int64_t p = indptr[i]; p < indptr[i + 1]; ++p) {
      const int64_t j = indices[p];
      const float* xj = X + j * ldx;
      double z = 0.0, za = 0.0, gd = 0.0, gda = 0.0;
      for (int32_t k = 0; k < d; ++k) {
        const double tz = (double)xi[k] * (double)xj[k];
        z += tz;
        za += fabs(tz);
        const double t = (double)gi[k] * (double)xj[k];
        gd += t;
        gda += fabs(t);
      }
      const double s = edge_f(op, z);
      const double a = values ? (double)values[p] : 1.0;
      const double dz = a * gd * edge_df(op, z);
      const double dzm = fabs(a) * gda * (fabs(edge_df(op, z)) + edge_l2(op) * za);
      double* oi = dX + i * (int64_t)d;
      double* oj = dX + j * (int64_t)d;
      for (int32_t k = 0; k < d; ++k) {
        oi[k] += dz * (double)xj[k];
        oj[k] += a * s * (double)gi[k] + dz * (double)xi[k];
      }
      if (mag) {
        double* mi = mag + i * (int64_t)d;
        double* mj = mag + j * (int64_t)d;
        for (int32_t k = 0; k < d; ++k) {
          mi[k] += dzm * fabs((double)xj[k]);
          mj[k] += fabs(a) * (fabs(s) + edge_l1(op) * za) * fabs((double)gi[k]) + dzm * fabs((double)xi[k]);
        }
      }
    }
  }
}

/* ---- other reductions of the sparse-dense product (Section 3.4, Section 3.5: reduce = 'sum',
 * 'mean', 'min', 'max') ----------------------------------------------------------------------
 * The paper names the reductions and gives no formula; the reading taken is the one of the
 * scatter-style reduce it refers to:
 *   mean: Y[i,k] = (sum_p a_p x_jk) / len_i, len_i = stored entries of row i; empty row -> 0.
 *   min / max: Y[i,k] = min / max over the stored entries p of row i of a_p * x_jk; arg[i,k] = the
 *     position p (index into the CSR arrays) of the first entry attaining it; empty row -> 0, arg -1.
 * For min / max the product is formed and compared in fp32 (one rounded multiply), the precision of
 * the method's arithmetic, so that the position (an integer decided by floating point) is decided in
 * the same precision on both sides and can be compared bit for bit.  Against the plain fp64 definition
 * this changes nothing in the value (rounding is monotone: the fp32 extremum is the fp64 extremum
 * rounded once) and moves the position only between entries whose products round to the same fp32
 * number; tests/test_oracle_scale_pins.py asserts exactly that against an fp64 brute force.
 * reduce: 1 mean, 2 min, 3 max.  arg may be NULL for mean.  mag (mean only, may be NULL) is the sum
 * of |a_p x_jk| / len_i. */
void isp_oracle_spmm_reduce(int64_t n_rows, const int64_t* indptr, const int32_t* indices, const float* values,
                            const float* X, int64_t ldx, int32_t d, int reduce, double* Y, int32_t* arg,
                            double* mag) {
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t i = 0; i < n_rows; ++i) {
    double* y = Y + i * (int64_t)d;
    const int64_t s = indptr[i], e = indptr[i + 1];
    if (reduce == 1) {
      double* m = mag ? mag + i * (int64_t)d : NULL;
      for (int32_t k = 0; k < d; ++k) {
        double acc = 0.0, am = 0.0;
        for (int64_t p = s; p < e; ++p) {
          const double t = (values ? (double)values[p] : 1.0) * (double)X[(int64_t)indices[p] * ldx + k];
          acc += t;
          am += fabs(t);
        }
        y[k] = e > s ? acc / (double)(e - s) : 0.0;
        if (m) m[k] = e > s ? am / (double)(e - s) : 0.0;
      }
    } else {
      int32_t* a = arg + i * (int64_t)d;
      for (int32_t k = 0; k < d; ++k) {
        float best = 0.0f;
        int32_t where = -1;
        for (int64_t p = s; p < e; ++p) {
          const float av = values ? values[p] : 1.0f;
          const volatile float t = av * X[(int64_t)indices[p] * ldx + k];  /* fp32 product */
          const float tv = t;
          if (where < 0 || (reduce == 2 ? tv < best : tv > best)) { best = tv; where = (int32_t)p; }
        }
        y[k] = (double)best;
        a[k] = where;
      }
    }
  }
}

/* Backward of the reductions above, scatter form (sequential), dX is n_cols x d, zeroed here:
 *   mean:      dX[j,:] += (a_p / len_i) dY[i,:]                for every entry p = (i, j)
 *   min / max: dX[col(p),k] += a_p dY[i,k]  with p = arg[i,k]  (nothing for arg = -1)        */
void isp_oracle_spmm_reduce_backward(int64_t n_rows, int64_t n_cols, const int64_t* indptr, const int32_t* indices,
                                     const float* values, const float* dY, int64_t ldg, int32_t d, int reduce,
                                     const int32_t* arg, double* dX, double* mag) {
  memset(dX, 0, (size_t)n_cols * (size_t)d * sizeof(double));
  if (mag) memset(mag, 0, (size_t)n_cols * (size_t)d * sizeof(double));
  for (int64_t i = 0; i < n_rows; ++i) {
    const int64_t s = indptr[i], e = indptr[i + 1];
    const float* g = dY + i * ldg;
    if (reduce == 1) {
      for (int64_t p = s; p < e; ++p) {
        const double w = (values ? (double)values[p] : 1.0) / (double)(e - s);
        double* o = dX + (int64_t)indices[p] * d;
        double* m = mag ? mag + (int64_t)indices[p] * d : NULL;
        for (int32_t k = 0; k < d; ++k) {
          o[k] += w * (double)g[k];
          if (m) m[k] += fabs(w * (double)g[k]);
        }
      }
    } else {
      for (int32_t k = 0; k < d; ++k) {
        const int32_t p = arg[i * (int64_t)d + k];
        if (p < 0) continue;
        const double t = (values ? (double)values[p] : 1.0) * (double)g[k];
        dX[(int64_t)indices[p] * d + k] += t;
        if (mag) mag[(int64_t)indices[p] * d + k] += fabs(t);
      }
    }
  }
}
