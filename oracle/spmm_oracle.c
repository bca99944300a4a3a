/*
 * TEST INFRASTRUCTURE -- the reference checker, not the product.
 *
 * Plain fp64 CPU evaluation of Y = A.X (and of A^l.X) over the ORIGINAL,
 * undecomposed CSR operand.  Only tests, the smoke check and the benchmark's
 * CPU-baseline leg may call this; the GPU library never does and shares no
 * code with it.
 *
 * What is computed is the order-2, single-term case of the paper's kernel
 * class (section "SpTTN Kernels": one sparse operand contracted with dense
 * operands, dense output): Y(i,c) = sum_j A(i,j) X(j,c).  The loop order is
 * the stored order of the sparse operand, row then nonzero (section
 * "SpTTN-Cyclops Framework": sparse indices are iterated in CSF order), with
 * the dense index innermost as a scaled vector update, the axpy leaf of the
 * figure "Loop nest for an order 4 TTMc kernel".  One such product costs
 * 2.nnz.k operations (section "Pairwise Contraction": 2.nnz(T).S for one
 * sparse-times-dense-matrix contraction).
 *
 * Inputs are the same fp32 bit patterns the GPU path receives, widened to
 * fp64; all accumulation is fp64.  Besides Y the routine returns the
 * magnitude bound  B = |A|.|X|  that the elementwise tolerance is scaled by.
 * Rows are independent, so the OpenMP loop over rows changes no summation
 * order.  No blocking, fusion or reordering.
 *
 * The file also holds the sampled dense-dense product on the same pattern (oracle_sddmm).
 *
 * Pins (tests/test_oracle_pins.py): dense brute force, identity /
 * permutation / diagonal operands, unit-vector columns, row-stochastic
 * operand times ones, grid operator times ones and its sine eigenvectors
 * (also for powers), and a library CSR product.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/*
 * Y[r, 0:kc] = sum_p vals[p] * X[colidx[p], 0:kc]   over the nonzeros p of row i,
 * B[r, 0:kc] = sum_p |vals[p]| * |X[colidx[p], 0:kc]|,
 * where i = rows[r] (or i = r when rows is NULL, nrows = n).
 * X is fp32 with leading dimension ldx (so a column slice is X + c0);
 * Y and B are fp64 with leading dimension kc.
 * Returns 0, or -1 on bad arguments.
 */
int oracle_spmm(int64_t n, const int64_t *rowptr, const int32_t *colidx,
                const float *vals, const float *X, int64_t ldx, int32_t kc,
                int64_t nrows, const int64_t *rows, double *Y, double *B) {
  if (n < 0 || !rowptr || (!colidx && rowptr[n] > 0) || (!vals && rowptr[n] > 0) ||
      !X || kc < 1 || ldx < kc || nrows < 0 || !Y || !B)
    return -1;
  if (!rows && nrows != n) return -1;
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t r = 0; r < nrows; ++r) {
    const int64_t i = rows ? rows[r] : r;
    double *y = Y + r * (int64_t)kc;
    double *bb = B + r * (int64_t)kc;
    for (int32_t c = 0; c < kc; ++c) { y[c] = 0.0; bb[c] = 0.0; }
    if (i < 0 || i >= n) continue; /* out-of-range selection: left at zero */
    for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
      const double a = (double)vals[p];
      const float *x = X + (int64_t)colidx[p] * ldx;
      for (int32_t c = 0; c < kc; ++c) {
        y[c] += a * (double)x[c];
        bb[c] += fabs(a) * fabs((double)x[c]);
      }
    }
  }
  return 0;
}

/*
 * Chained products kept in fp64 throughout:
 *   X_0 = X (widened), E_0 = |X|;  X_{t+1} = A.X_t,  E_{t+1} = |A|.E_t,  t < l.
 * Writes X_l to Xl and E_l to El (both n x k fp64, contiguous).
 * Returns 0, -1 on bad arguments, -2 when out of memory.
 */
int oracle_spmm_iter(int64_t n, const int64_t *rowptr, const int32_t *colidx,
                     const float *vals, const float *X, int32_t k, int32_t l,
                     double *Xl, double *El) {
  if (n < 0 || !rowptr || (!colidx && rowptr[n] > 0) || (!vals && rowptr[n] > 0) ||
      !X || k < 1 || l < 0 || !Xl || !El)
    return -1;
  const int64_t tot = n * (int64_t)k;
  for (int64_t q = 0; q < tot; ++q) { Xl[q] = (double)X[q]; El[q] = fabs((double)X[q]); }
  if (l == 0) return 0;
  double *Xn = (double *)malloc((size_t)(tot > 0 ? tot : 1) * sizeof(double));
  double *En = (double *)malloc((size_t)(tot > 0 ? tot : 1) * sizeof(double));
  if (!Xn || !En) { free(Xn); free(En); return -2; }
  for (int32_t t = 0; t < l; ++t) {
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n; ++i) {
      double *y = Xn + i * (int64_t)k;
      double *e = En + i * (int64_t)k;
      for (int32_t c = 0; c < k; ++c) { y[c] = 0.0; e[c] = 0.0; }
      for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
        const double a = (double)vals[p];
        const double *x = Xl + (int64_t)colidx[p] * k;
        const double *ex = El + (int64_t)colidx[p] * k;
        for (int32_t c = 0; c < k; ++c) {
          y[c] += a * x[c];
          e[c] += fabs(a) * ex[c];
        }
      }
    }
    memcpy(Xl, Xn, (size_t)tot * sizeof(double));
    memcpy(El, En, (size_t)tot * sizeof(double));
  }
  free(Xn); free(En);
  return 0;
}

/*
 * Sampled dense-dense product on the pattern of A (the order-2 case of the paper's TTTP kernel,
 * section "Tensor Decomposition and Completion Algorithms", with the third mode dropped; the
 * output has the sparsity of the sparse operand, section "SpTTN Kernels"):
 *   S[p] = vals[p] * sum_r U[i, r] * V[j, r]        for the nonzero p = (i, j) of A,
 *   B[p] = |vals[p]| * sum_r |U[i, r]| * |V[j, r]|   (the bound the tolerance is scaled by),
 * in CSR order of A, fp64 accumulation over r in increasing order.  U, V: n x k fp32 row-major.
 * Returns 0, or -1 on bad arguments.
 */
int oracle_sddmm(int64_t n, const int64_t *rowptr, const int32_t *colidx, const float *vals,
                 const float *U, const float *V, int32_t k, double *S, double *B) {
  if (n < 0 || !rowptr || (!colidx && rowptr[n] > 0) || (!vals && rowptr[n] > 0) || !U || !V ||
      k < 1 || !S || !B)
    return -1;
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t i = 0; i < n; ++i) {
    const float *u = U + i * (int64_t)k;
    for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
      const float *v = V + (int64_t)colidx[p] * k;
      double dot = 0.0, adot = 0.0;
      for (int32_t r = 0; r < k; ++r) {
        dot += (double)u[r] * (double)v[r];
        adot += fabs((double)u[r]) * fabs((double)v[r]);
      }
      S[p] = (double)vals[p] * dot;
      B[p] = fabs((double)vals[p]) * adot;
    }
  }
  return 0;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
