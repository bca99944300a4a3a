/*
 * arrow.h -- C boundary of the arrow-matrix-decomposition SpMM library for one
 * MI355X (gfx950).
 *
 * The operation.  For a square sparse A (n x n, CSR, fp32) and a tall-skinny
 * dense X (n x k, fp32, row-major) the library computes Y = A.X, the order-2,
 * single-term member of the kernel class of the paper's section "SpTTN
 * Kernels" (one sparse operand contracted with dense operands into a dense
 * output); CSR is the order-2 case of the storage of section "Tensor Sparsity
 * and Sparse Storage".  One product is counted as 2.nnz.k operations (section
 * "Pairwise Contraction").  The product is not evaluated on A directly but as
 *
 *        Y = sum_{i < L}  P_i^T . B_i . (P_i . X)
 *
 * where (P_i X)[p,:] = X[perm_i[p],:] selects and reorders n_i <= n rows, and
 * every B_i is an ARROW MATRIX of width b: a stored entry (p,q) of B_i has
 * p/b == q/b (diagonal block), or p < b (first block row, the "head" rows), or
 * q < b (first block column).  The paper itself does not define this
 * decomposition; the definition used here is: the head of a level holds the
 * highest-degree vertices of what is still unassigned (plus block separators
 * when they make the level complete), the rest are laid out by a linear
 * arrangement and cut into blocks of b; entries that fit the arrow shape
 * belong to the level, all others go on to the next level.  Each nonzero of A
 * lands in exactly one level, unchanged.
 *
 * Conventions.
 *  - "host" pointers are ordinary CPU memory, "device" pointers are HIP device
 *    memory of the current device.  The library allocates no device memory:
 *    the caller provides the image buffer and the workspace and keeps them
 *    alive until arrow_destroy().
 *  - X and Y are contiguous row-major with leading dimension k and must be
 *    16-byte aligned.  Y is overwritten (never accumulated into).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Compute calls only enqueue work on it and return without synchronising.
 *    A handle may be used from one stream at a time.
 *  - Every call returns ARROW_OK (0) or a negative arrow_status; nothing
 *    throws or aborts.  arrow_last_error() gives a thread-local description
 *    of the last failure.
 */
#ifndef ARROW_H
#define ARROW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum arrow_status {
  ARROW_OK = 0,
  ARROW_EINVAL = -1,    /* bad argument: n<=0, b<=0, k<=0, l<0, NULL, malformed CSR */
  ARROW_ENOMEM = -2,    /* host allocation failed                                   */
  ARROW_ENOTREADY = -3, /* compute call before arrow_upload / arrow_set_workspace   */
  ARROW_ETOOSMALL = -4, /* a caller-provided buffer is smaller than required        */
  ARROW_EHIP = -5,      /* a HIP runtime call failed (text in arrow_last_error)     */
  ARROW_EINTERNAL = -6  /* a self-check of the decomposition failed                 */
} arrow_status;

typedef struct arrow_handle arrow_handle; /* opaque, host memory, owned by the library */

/* Whole-decomposition figures. */
typedef struct arrow_info_t {
  int64_t n;          /* rows = columns of A                         */
  int64_t nnz;        /* stored entries of A                         */
  int32_t b;          /* arrow width                                 */
  int32_t levels;     /* L, number of arrow matrices                 */
  int64_t max_chunks; /* largest number of head partials of a level  */
  double decompose_seconds;
} arrow_info_t;

/* Figures of one level i. Regions partition the stored entries of B_i. */
typedef struct arrow_level_info_t {
  int64_t n_i;          /* active vertices = length of perm_i                    */
  int64_t nnz;          /* stored entries of B_i                                 */
  int64_t nnz_head_head;/* p < b and q < b                                       */
  int64_t nnz_head_row; /* p < b and q >= b  (first block row, off the corner)   */
  int64_t nnz_head_col; /* p >= b and q < b  (first block column)                */
  int64_t nnz_diag;     /* p >= b and q >= b (then p/b == q/b)                   */
  int64_t short_rows;   /* items handled one per lane group (short rows, class pieces) */
  int64_t chunks;       /* items (chunks of long rows) handled one per wavefront */
  int64_t split_rows;   /* rows whose chunks are combined by the reduction pass  */
  int64_t partials;     /* partial vectors those rows produce (one per chunk)    */
  int64_t nnz_rows;     /* entries held by the lane-group row list               */
  int64_t nnz_chunks;   /* entries held by the chunk list                        */
  int64_t x_rows_rows;  /* distinct rows of X the row list reads                 */
  int64_t x_rows_chunks;/* distinct rows of X the chunk list reads               */
  int64_t window_tiles; /* diagonal-block tiles run with their X window in LDS   */
  int64_t window_rows;  /* rows those tiles cover                                */
  int64_t nnz_window;   /* entries of those rows                                 */
  int64_t rows_partials;  /* lane-group items that write a partial vector        */
  int64_t chunks_partials;/* wavefront items that write a partial vector         */
  int64_t panel_rows;   /* head rows whose head-block entries run in panels (accumulators in LDS) */
  int64_t panel_bins;   /* lane-group entry streams of those panels              */
  int64_t nnz_panel;    /* entries held by the panels                            */
  int32_t blocks;       /* ceil(n_i / b)                                         */
  int32_t separator_rule; /* 1 if block separators were promoted into the head   */
  int64_t nnz_fused;    /* level 0 only: entries of later levels that the packed image lists with the
                           level-0 rows of their vertices (fused levels); the work-list figures above
                           (nnz_rows, nnz_chunks, nnz_window, nnz_panel) then add up to nnz + nnz_fused,
                           and those of the later levels are 0 */
  int64_t corner;       /* rows = columns of the dense corner of the head block run in LDS tiles (0 = none) */
  int64_t corner_tiles; /* non-empty 256 x 256 tiles of the corner                            */
  int64_t corner_items; /* work items (runs of tiles of one row panel) of the corner kernel   */
  int64_t nnz_corner;   /* entries held by the corner tiles                                   */
} arrow_level_info_t;

/* Per-kernel-class time of the last profiled product, milliseconds. */
typedef struct arrow_profile_t {
  float rows_ms;    /* lane-group-per-row kernel (first block column + diagonal blocks, short head rows) */
  float chunks_ms;  /* wavefront-per-chunk kernel (head rows and other long rows)                         */
  float reduce_ms;  /* cross-chunk reduction + scatter                                                    */
  float stage_ms;  /* gather of the head rows X_0 into the contiguous staging buffer                      */
  float window_ms;  /* diagonal-block tiles with the X window staged in LDS                               */
  float total_ms;   /* first launch to last launch of the product                                         */
  int32_t rows_launches, chunks_launches, reduce_launches, stage_launches, window_launches; /* launches per class (one per level that has such work) */
  float panel_ms;   /* head panels: head-block entries of sparse head rows, accumulators in LDS          */
  int32_t panel_launches;
  float corner_ms;  /* dense corner of the head block: LDS tiles + the pass that adds their results to Y */
  int32_t corner_launches;
} arrow_profile_t;

/*
 * Decompose A into arrow matrices of width b (host only, no GPU needed).
 *   n        rows = columns, 1 <= n <= 2^31 - 2
 *   rowptr   host, n+1 entries, rowptr[0] == 0, non-decreasing, rowptr[n] = nnz < 2^32 - 1
 *   colidx   host, nnz entries in [0,n), strictly increasing inside every row
 *   vals     host, nnz fp32 values (explicit zeros are kept as entries)
 *   b        arrow width >= 1 (b >= n gives one level with B_0 = A reordered)
 *   out      receives the handle; the CSR arrays are not referenced after return
 * Errors: ARROW_EINVAL (any violated condition above), ARROW_ENOMEM.
 */
int arrow_decompose(int64_t n, const int64_t *rowptr, const int32_t *colidx,
                    const float *vals, int32_t b, arrow_handle **out);

/* Bytes of device memory the packed image (tiles, work lists, permutations) needs. 0 if h is NULL. */
size_t arrow_device_bytes(const arrow_handle *h);

/*
 * Copy the packed image into caller-owned device memory (256-byte aligned,
 * at least arrow_device_bytes(h)) with an asynchronous copy on `stream`, and
 * bind the handle to it.  The source is the handle's pageable host copy, so the
 * call may block until the copy has been staged.  Errors: EINVAL, ETOOSMALL, EHIP.
 */
int arrow_upload(arrow_handle *h, void *dev_buf, size_t bytes, void *stream);

/*
 * Device workspace a product with k columns needs: head partials of the
 * largest level, the staged head rows, the results of the corner and panel
 * work items, plus one n x k buffer for the chained products of
 * arrow_spmm_iter.  arrow_set_workspace binds caller-owned device memory
 * (256-byte aligned); it may be rebound at any time the stream is idle.
 */
size_t arrow_workspace_bytes(const arrow_handle *h, int32_t k);
int arrow_set_workspace(arrow_handle *h, void *dev_ws, size_t bytes);

/*
 * Y = A.X = sum_i P_i^T B_i (P_i X).   X, Y: device, n x k fp32, must not overlap.
 * Level 0 stores every row of Y (perm_0 is a full permutation); later levels
 * add into the rows they touch, in stream order, so the result does not
 * depend on scheduling (no floating-point atomics are used).
 * With profiling off the call only launches kernels on `stream` (no allocation, no memset, no
 * synchronisation), so it may be recorded into a HIP graph by a caller that captures `stream`;
 * the same holds for arrow_spmm_iter (plus one device-to-device copy for odd l) and arrow_sddmm.
 * Errors: EINVAL (NULL, k < 1, misaligned; the byte ranges of X and Y overlap each other or the
 * bound workspace, or Y overlaps the device image), ENOTREADY, ETOOSMALL (workspace bound for a
 * smaller k), EHIP.
 */
int arrow_spmm(arrow_handle *h, const float *X, float *Y, int32_t k, void *stream);

/*
 * arrow_spmm for callers that cannot allocate or own device scratch memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same product, same kernels and
 * same results bit for bit as arrow_spmm, but the partial vectors and the staged head rows live
 * in a device array of ARROW_STATIC_SCRATCH_BYTES that is part of the library itself (one copy
 * per GPU, held until the process ends), so no workspace has to be bound (arrow_upload must have
 * run on the current device).  The call allocates nothing, records no events even when profiling
 * is on, and only launches kernels on `stream`.
 *   X, Y    DEVICE, n x k fp32 row-major, 16-byte aligned, must not overlap; Y is overwritten
 * The scratch need is arrow_workspace_bytes(h, k) minus the n x k buffer of the chained products
 * (partial vectors of the largest level + min(b, n) staged head rows of k floats); if it exceeds
 * the array the call fails with ARROW_ETOOSMALL and nothing is launched.  All calls on one GPU
 * share that GPU's array, whatever the handle or stream: calls that overlap in time on one GPU
 * race and give wrong results; calls in stream order are safe.  Nothing in the array has to start
 * at zero (every slot a product reads was written earlier in the same product), so the previous
 * call's contents do not matter.
 * Errors: EINVAL (NULL, k < 1, overlapping X and Y, alignment), ENOTREADY (no image), ETOOSMALL, EHIP.
 */
#define ARROW_STATIC_SCRATCH_BYTES (64u << 20)
int arrow_spmm_static(arrow_handle *h, const float *X, float *Y, int32_t k, void *stream);

/*
 * X <- A^l . X, l chained products rounded to fp32 after each one, result left
 * in X (l = 0 leaves X untouched).  Uses the n x k part of the workspace.
 * Errors as arrow_spmm, plus EINVAL for l < 0.
 */
int arrow_spmm_iter(arrow_handle *h, float *X, int32_t k, int32_t l, void *stream);

/*
 * The permutation gather of one level on its own: Xp[p,:] = X[perm_i[p],:]
 * for p < n_i.  X: device n x k; Xp: device n_i x k.  The products above fuse
 * this step into their loads; it is exported for layouts that want P_i X
 * materialised and for testing.  Errors: EINVAL, ENOTREADY, EHIP.
 */
int arrow_gather(arrow_handle *h, int32_t level, const float *X, float *Xp,
                 int32_t k, void *stream);

/* Introspection (host only). */
int arrow_info(const arrow_handle *h, arrow_info_t *out);
int arrow_level_info(const arrow_handle *h, int32_t level, arrow_level_info_t *out);

/*
 * Host copies of one level for checking: perm (n_i entries, position ->
 * original vertex) and the stored entries of B_i as coordinate triples in
 * position space (rows/cols/vals, nnz_i entries each).  Any output pointer may
 * be NULL to skip it.  Errors: EINVAL.
 */
int arrow_export_level(const arrow_handle *h, int32_t level, int32_t *perm,
                       int32_t *rows, int32_t *cols, float *vals);

/*
 * Host-only consistency check of the packed device image against the levels it was built from:
 * offsets ordered and in range, row ids inside X / the staging buffer / the LDS windows, every
 * partial slot written once, every row of every level produced exactly once from exactly its
 * entries, the entry map a bijection that keeps row and value; with fused levels the execution
 * form (later levels' entries listed with the level-0 rows) is rebuilt and compared entry by entry
 * with the levels first; panel streams and corner tiles (items and panels partition the tiles,
 * runs ordered and never sharing a row) are covered as well.
 * Returns ARROW_OK or ARROW_EINTERNAL (text in arrow_last_error).  O(nnz log nnz), no GPU.
 */
int arrow_self_check(const arrow_handle *h);

/*
 * Every choice the decomposition, the packing of the device image and the launches leave open,
 * as one plain struct.  arrow_options_default() fills it with the built-in defaults (given per
 * field below) and then applies overrides from the environment: a variable ARROW_<FIELD NAME IN
 * CAPITALS> holding a decimal integer replaces that field (the two ratios are given as
 * ARROW_WINDOW_REUSE_X10 = 10 x window_reuse and ARROW_WINDOW_SHARE_X1000 = 1000 x
 * window_level_share).  The environment is read by that one function and nowhere else; it exists
 * for experiments and tests.  arrow_decompose(...) and arrow_load(...) are
 * arrow_decompose_with(..., NULL, ...) and arrow_load_with(..., NULL, ...): NULL options mean
 * "what arrow_options_default() returns now".
 */
typedef struct arrow_options_t {
  /* --- decomposition (host) --- */
  int32_t separators;     /* 1: try the block-separator rule before the plain top-degree head     */
  int32_t bfs_tail;       /* 1: later levels / the body of a plain level are arranged by traversal */
  int32_t head_by_id;     /* 1: head vertices of the plain rule in id order; 0: by falling degree  */
  int64_t hubs_first;     /* 0: with head_by_id, this many highest degrees lead the head by falling
                             degree (makes the top-left corner of the head block dense)            */
  /* --- packing of the device image (host) --- */
  int32_t short_max;      /* 16: rows with at most this many entries go to the lane-group list    */
  int32_t chunk_nnz;      /* 256: most entries of a wavefront chunk                               */
  int32_t chunk_min;      /* 64: column windows of a row are merged until a piece holds this many */
  int32_t window_rows;    /* 4096: column positions per window of the chunk order (0 = row-major) */
  int32_t classes;        /* 0: column classes of the die queues (rounded up to a multiple of 8)   */
  int32_t class_gran;     /* 512: column positions dealt to a class at a time                     */
  int32_t class_min;      /* 32: a row is split by class when it holds classes x this many entries */
  int32_t piece_max;      /* 48: a piece of a long row with at most this many entries is a lane-group item */
  int32_t stage_head;     /* 1: gather the head rows of level 0 into a contiguous buffer per product */
  int32_t stage_short;    /* -1: short rows read head columns from that buffer when the head is
                             scattered over X; 1 / 0: always / never                               */
  int32_t empty_last;     /* 1: level-0 rows without entries are listed after all other short rows */
  int32_t panel;          /* 0: head panels (128 head rows per group, accumulators in LDS, one column
                             class per accelerator die) for head rows with few entries per window  */
  int32_t panel_min;      /* 8: fewest head-block entries of a row that joins a panel             */
  int32_t window_span;    /* 2048: widest column span of a diagonal-block tile whose window of
                             P_i X is staged in LDS (at most 4096; 0 = no such tiles)               */
  int32_t window_tile_rows; /* 1024: most rows of such a tile                                      */
  double window_reuse;    /* 8.0: a tile is kept when its diagonal-block entries >= this x its span */
  double window_level_share; /* 0.05: ... and the tiles of a level when they hold this share of it */
  int32_t fuse_levels;    /* 1: the entries later levels hold for a vertex are listed with its
                             level-0 row: one item sums over all arrow matrices, later levels need
                             neither launches nor a read-modify-write of Y; 0: one launch set per level */
  int32_t corner;         /* 0: 1 = rows and columns [0, S) of the head block of level 0 run in tiles
                             of 256 x 256 with staged head rows and accumulators in LDS              */
  int32_t corner_max;     /* 65536: largest S considered                                          */
  int32_t corner_min_tile;/* 768: S is the largest multiple of 256 whose outermost band of tiles
                             holds this many entries per tile on average                            */
  /* --- launches (may also be changed later with arrow_set_option) --- */
  int32_t kc;             /* 0 = automatic (64 when the head is staged and k > 64, else the whole
                             row up to 256 columns): columns per pass of the chunk kernel           */
  int64_t l2_resident_bytes; /* 2 MiB: share of a die's L2 a resident slice of the staged head may
                             take when kc is chosen automatically with die queues                   */
} arrow_options_t;

/* Built-in defaults, then the ARROW_* environment overrides described above. NULL is ignored. */
void arrow_options_default(arrow_options_t *opt);

/*
 * arrow_decompose / arrow_load with explicit options (opt == NULL: arrow_options_default()).
 * arrow_repack rebuilds the device image of an existing handle with other packing and launch
 * options (the decomposition fields are ignored: the levels stay as they are); the handle is
 * unbound from its device image and workspace and needs arrow_upload and arrow_set_workspace
 * again.  Errors as arrow_decompose / arrow_load.
 */
int arrow_decompose_with(int64_t n, const int64_t *rowptr, const int32_t *colidx, const float *vals,
                         int32_t b, const arrow_options_t *opt, arrow_handle **out);
int arrow_load_with(const char *path, const arrow_options_t *opt, arrow_handle **out);
int arrow_repack(arrow_handle *h, const arrow_options_t *opt);

/*
 * Launch-time tunables of an existing handle, by name:
 *   "kc"        columns per pass of the chunk kernel; a smaller slice shrinks the working set of
 *               X rows per pass and re-reads the entries k/kc times.  0 = automatic: 64 when the
 *               head is staged and k > 64, the whole row (up to 256 columns) otherwise
 *   "l2_resident_bytes"  share of one die's 4 MiB L2 that a resident slice of the staged head
 *               may take when kc is chosen automatically (default 2 MiB)
 *   "sddmm_image_order"  1: arrow_sddmm writes S in the order of the packed image instead of the
 *               caller's CSR order (contiguous stores; arrow_export_entry_map tells which nonzero
 *               each element belongs to); default 0
 * Errors: EINVAL (unknown name, value out of range).
 */
int arrow_set_option(arrow_handle *h, const char *name, int64_t value);

/*
 * Profiling: when enabled, every product brackets its launches with HIP
 * events on the caller's stream; arrow_get_profile waits for them and
 * reports per-kernel-class times of the most recent product.
 */
int arrow_set_profiling(arrow_handle *h, int32_t enabled);
int arrow_get_profile(arrow_handle *h, arrow_profile_t *out);
/* Same, restricted to the launches of one level (level < 0: all levels; total_ms always spans
 * the whole product). */
int arrow_get_level_profile(arrow_handle *h, int32_t level, arrow_profile_t *out);

/*
 * Sampled dense-dense product on the pattern of A,
 *     S[p] = a_p * sum_r U[i, r] V[j, r]        for the nonzero p = (i, j) of A,
 * the order-2 case of the paper's TTTP kernel (section "Tensor Decomposition and Completion
 * Algorithms"; the output has the sparsity of the sparse operand, section "SpTTN Kernels").  It
 * runs over the same arrow layout and work lists as the product: the rows V[j, :] are gathered
 * exactly as the rows X[j, :] of arrow_spmm are, U[i, :] takes the place of the accumulator.
 *
 * The kernels need the entry map (one uint32 per nonzero: image order -> index in the caller's
 * CSR arrays).  arrow_sddmm_device_bytes returns its size; arrow_sddmm_upload copies it to
 * `dev_buf` (DEVICE memory, 256-byte aligned, caller-owned, must outlive every arrow_sddmm call on
 * the handle) asynchronously on `stream`.
 *
 * arrow_sddmm: U, V DEVICE pointers to n x k fp32 row-major, 16-byte aligned (U == V is allowed);
 * S DEVICE pointer to nnz fp32, written in the order of the caller's CSR arrays (every element is
 * written exactly once, nothing is accumulated).  Needs arrow_upload, arrow_sddmm_upload and a
 * workspace of arrow_workspace_bytes(h, k).  Launches on `stream` and returns without waiting.
 * fp32 arithmetic, deterministic summation order.
 * arrow_export_entry_map copies the entry map to `out` (HOST, nnz uint32): element e of an
 * image-order S (option "sddmm_image_order") is the nonzero out[e] of the caller's CSR arrays.
 * Errors: EINVAL (NULL, alignment, k < 1), ENOTREADY (no image / map / workspace), ETOOSMALL
 * (buffer or workspace too small), EHIP.
 */
size_t arrow_sddmm_device_bytes(const arrow_handle *h);
int arrow_sddmm_upload(arrow_handle *h, void *dev_buf, size_t bytes, void *stream);
int arrow_sddmm(arrow_handle *h, const float *U, const float *V, float *S, int32_t k, void *stream);
int arrow_export_entry_map(const arrow_handle *h, uint32_t *out);

/*
 * Persistence (host only).  arrow_save writes the arrow matrices of a handle (permutations and
 * the entries of every B_i with their indices in the caller's CSR arrays, not the device image)
 * to `path`; arrow_load reads such a file, checks it (sizes, injective permutations, ordered
 * in-range column positions, arrow shape of width b, entry count, source indices a bijection onto
 * the nonzeros) and rebuilds the device image with the loader's packing options
 * (arrow_load_with), so a decomposition is paid once per operand.  The loaded handle behaves like one
 * from arrow_decompose (it still needs arrow_upload and a workspace).
 * Errors: EINVAL (NULL, file cannot be opened / written, not a level file, truncated, fails a
 * check), ENOMEM.
 */
int arrow_save(const arrow_handle *h, const char *path);
int arrow_load(const char *path, arrow_handle **out);

/*
 * Measurement aid (no handle, not part of a product): a bare gather of whole rows, the yardstick
 * the product kernels' gather rates are quoted against.  `gathers` pseudo-random rows (a fixed
 * sequence) of the row-major fp32 matrix X (DEVICE, x_rows x k, 16-byte aligned) are read with one
 * 16-byte load per lane, eight rows in flight per lane group, and summed.  The rows are drawn from
 * the first region_rows rows of X; with per_die != 0 every accelerator die draws from a region of
 * its own (die d: rows [d * region_rows, (d + 1) * region_rows)), so a small region stays in that
 * die's L2; with from_lds != 0 the region (at most 64 KiB) is copied into LDS first and the rows
 * are read from there.  k must be a power of two in [4, 256].  `out` (DEVICE, at least
 * arrow_probe_gather_out_bytes(gathers) bytes) receives per-lane sums nobody needs.  Launches one
 * kernel on `stream` and returns; the caller times it.
 * Errors: EINVAL, ETOOSMALL, EHIP.
 */
size_t arrow_probe_gather_out_bytes(int64_t gathers);
int arrow_probe_gather(const float *X, int64_t x_rows, int32_t k, int64_t region_rows, int32_t per_die,
                       int32_t from_lds, int64_t gathers, float *out, size_t out_bytes, void *stream);

/* Thread-local text of the last error ("" if none). Never NULL. */
const char *arrow_last_error(void);

/* Release the handle and its host memory (not the caller's device buffers). NULL is ignored. */
void arrow_destroy(arrow_handle *h);

#ifdef __cplusplus
}
#endif
#endif /* ARROW_H */
