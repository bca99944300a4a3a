/*
 * Order-3 MTTKRP on one MI355X (gfx950), C boundary.
 *
 *     A(i, a) = sum_{j,k} T(i, j, k) * B(j, a) * C(k, a)
 *
 * the matricized-tensor times Khatri-Rao product of the paper (MTTKRP equation, section "Tensor
 * Decomposition and Completion Algorithms"), evaluated in the factorize-and-fuse form the paper
 * recommends for it (sections "Pairwise Contraction" and "Performance Evaluation": first the
 * fibre sums x(a) = sum_k T(i,j,k) C(k,a), then A(i,a) += x(a) B(j,a), fused in one loop nest so
 * the intermediate is a register vector), over T stored as compressed sparse fibres (section
 * "Tensor Sparsity and Sparse Storage": slices i, fibres (i, j), entries k).
 *
 * Host pointers and device pointers are marked per argument.  The library allocates no device
 * memory: image and workspace are the caller's.  All functions return an arrow_status code
 * (arrow.h); csf3_last_error() gives the text.  fp32 arithmetic, no atomics: results are bitwise
 * reproducible.  There is no CPU fallback.
 */
#ifndef CSF3_H
#define CSF3_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct csf3_handle csf3_handle; /* opaque, host memory, owned by the library */

typedef struct csf3_info_t {
  int64_t I, J, K;     /* mode sizes                                                        */
  int64_t nnz;         /* stored entries (duplicates of a coordinate are kept and so summed) */
  int64_t slices;      /* distinct i with at least one entry                                 */
  int64_t fibers;      /* distinct (i, j)                                                    */
  int64_t segments;    /* fibres cut into runs of at most 64 entries                         */
  int64_t items;       /* work items (one per wavefront): runs of segments of one slice      */
  int64_t split_rows;  /* slices cut into several items, combined by the reduction pass      */
  int64_t partials;    /* partial vectors those slices produce                               */
  int64_t distinct_j, distinct_k; /* rows of B / C the tensor references                    */
  double build_seconds;
} csf3_info_t;

/*
 * Build the compressed-sparse-fibre image of T for the mode-0 product (host only).
 *   I, J, K   mode sizes, 1 <= each <= 2^31 - 1 (indices are int32)
 *   nnz       entries, 0 <= nnz < 2^32 - 1
 *   ti,tj,tk  HOST, nnz coordinates each, 0 <= ti < I, 0 <= tj < J, 0 <= tk < K, any order
 *   tv        HOST, nnz fp32 values
 * The arrays are not referenced after return.  A product for another mode is obtained by passing
 * the coordinate arrays in another order.  Errors: EINVAL, ENOMEM.
 */
int csf3_build(int64_t I, int64_t J, int64_t K, int64_t nnz, const int32_t *ti, const int32_t *tj,
               const int32_t *tk, const float *tv, csf3_handle **out);

/* Bytes of DEVICE memory the image needs; csf3_upload copies it (256-byte aligned buffer,
 * asynchronous on `stream`) and binds the handle to it.  Errors: EINVAL, ETOOSMALL, EHIP. */
size_t csf3_device_bytes(const csf3_handle *h);
int csf3_upload(csf3_handle *h, void *dev_buf, size_t bytes, void *stream);

/* DEVICE workspace for rank R (partial vectors of split slices); 256-byte aligned. */
size_t csf3_workspace_bytes(const csf3_handle *h, int32_t R);
int csf3_set_workspace(csf3_handle *h, void *dev_ws, size_t bytes);

/*
 * A = MTTKRP(T; B, C).  B: DEVICE J x R, C: DEVICE K x R, A: DEVICE I x R, fp32 row-major,
 * 16-byte aligned; A is overwritten (rows of empty slices become 0) and must not overlap B or C.
 * Launches on `stream` (a hipStream_t) and returns without waiting.
 * Errors: EINVAL, ENOTREADY (no image / workspace), ETOOSMALL (workspace), EHIP.
 */
int csf3_mttkrp(csf3_handle *h, const float *B, const float *C, float *A, int32_t R, void *stream);

int csf3_info(const csf3_handle *h, csf3_info_t *out);

/*
 * Profiling: when enabled, csf3_mttkrp brackets its two launches with HIP events on the caller's
 * stream; csf3_get_profile waits for them and returns the times of the most recent product in
 * milliseconds (the fibre kernel, and the reduction over the partial vectors of split slices).
 * Errors: EINVAL, ENOTREADY (no profiled product has run), EHIP.
 */
int csf3_set_profiling(csf3_handle *h, int32_t enabled);
int csf3_get_profile(csf3_handle *h, float *kernel_ms, float *reduce_ms);

/* Thread-local text of the last error of a csf3_* call ("" if none). Never NULL. */
const char *csf3_last_error(void);

/* Release the handle and its host memory (not the caller's device buffers). NULL is ignored. */
void csf3_destroy(csf3_handle *h);

#ifdef __cplusplus
}
#endif
#endif /* CSF3_H */
