/*
 * TEST INFRASTRUCTURE -- the reference checker of the order-3 MTTKRP, not the product.
 *
 * Plain fp64 CPU evaluation of the matricized-tensor times Khatri-Rao product
 *     A(i, a) = sum_{j,k} T(i, j, k) * B(j, a) * C(k, a)
 * (the paper's MTTKRP equation, section "Tensor Decomposition and Completion Algorithms") over
 * the coordinate list of T, written out as that definition: one pass over the stored entries in
 * the order given, all three operands multiplied in the innermost statement (the form the
 * section "Unfactorized Contraction" describes), no intermediate, no blocking, no reordering.
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call this; the GPU
 * library never does and shares no code with it.
 *
 * Inputs are the same fp32 bit patterns the GPU path receives, widened to fp64; accumulation
 * is fp64.  Besides A the routine returns the magnitude bound
 *     E(i, a) = sum_{j,k} |T(i, j, k)| * |B(j, a)| * |C(k, a)|
 * that the elementwise tolerance is scaled by.
 * When the entries are sorted by i (non-decreasing), threads take disjoint ranges of i, so every
 * element of A is still summed by one thread in the order of the list; otherwise one thread runs.
 *
 * Pins (tests/test_oracle_pins.py): exact rational brute force, a hand-worked 2 x 2 x 2 case
 * (tests/golden), a dense library contraction, the all-ones tensor's closed form, mode sums
 * through indicator factors, the K = 1 case against the matrix-product checker, the pairwise
 * (factorized) evaluation, and index / factor swaps.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* first position p in [0, nnz) with idx[p] >= v (idx non-decreasing) */
static int64_t lower_bound_i32(const int32_t *idx, int64_t nnz, int64_t v) {
  int64_t lo = 0, hi = nnz;
  while (lo < hi) {
    const int64_t mid = lo + (hi - lo) / 2;
    if ((int64_t)idx[mid] < v) lo = mid + 1; else hi = mid;
  }
  return lo;
}

/*
 * T: nnz entries (ti[p], tj[p], tk[p], tv[p]) with 0 <= ti < I, 0 <= tj < J, 0 <= tk < K.
 * B: J x R, C: K x R, fp32 row-major.  A, E: I x R fp64 row-major, overwritten.
 * Returns 0, -1 on bad arguments, -2 when an index is out of range.
 */
int oracle_mttkrp(int64_t I, int64_t J, int64_t K, int64_t nnz, const int32_t *ti,
                  const int32_t *tj, const int32_t *tk, const float *tv, const float *B,
                  const float *C, int32_t R, double *A, double *E) {
  if (I < 1 || J < 1 || K < 1 || nnz < 0 || R < 1 || !B || !C || !A || !E ||
      (nnz > 0 && (!ti || !tj || !tk || !tv)))
    return -1;
  int sorted = 1;
  for (int64_t p = 0; p < nnz; ++p) {
    if (ti[p] < 0 || ti[p] >= I || tj[p] < 0 || tj[p] >= J || tk[p] < 0 || tk[p] >= K) return -2;
    if (p > 0 && ti[p - 1] > ti[p]) sorted = 0;
  }
  memset(A, 0, sizeof(double) * (size_t)I * (size_t)R);
  memset(E, 0, sizeof(double) * (size_t)I * (size_t)R);
  int parts = 1;
#ifdef _OPENMP
  if (sorted) parts = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(static, 1) num_threads(parts)
  for (int t = 0; t < parts; ++t) {
    const int64_t p0 = parts == 1 ? 0 : lower_bound_i32(ti, nnz, I * t / parts);
    const int64_t p1 = parts == 1 ? nnz : lower_bound_i32(ti, nnz, I * (t + 1) / parts);
    for (int64_t p = p0; p < p1; ++p) {
      const double v = (double)tv[p];
      const float *b = B + (int64_t)tj[p] * R;
      const float *c = C + (int64_t)tk[p] * R;
      double *a = A + (int64_t)ti[p] * R;
      double *e = E + (int64_t)ti[p] * R;
      for (int32_t r = 0; r < R; ++r) {
        a[r] += v * (double)b[r] * (double)c[r];
        e[r] += fabs(v) * fabs((double)b[r]) * fabs((double)c[r]);
      }
    }
  }
  return 0;
}
