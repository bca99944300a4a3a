// HIP kernels for gfx950 (CDNA4, 64-wide wavefronts) of the arrow SpMM
//     Y = sum_i P_i^T B_i (P_i X).
//
// Every kernel keeps the dense index innermost and contiguous across lanes:
// one stored entry a(p,q) triggers one scaled vector update
//     acc[0:k] += a * X[perm[q], 0:k]
// which is the axpy leaf of the paper's loop nests (figure "Loop nest for an
// order 4 TTMc kernel") at order 2, with rows then nonzeros as outer loops
// (section "SpTTN-Cyclops Framework": sparse indices in stored order).  The
// row gather P_i X is fused into the loads: entries carry perm[q] directly
// (or the row of the staged head buffer).  The scatter P_i^T is fused into the
// epilogue: results go to row perm[p] of Y.
//
// A lane owns VEC consecutive columns; LPR lanes ("a lane group") cover one
// slice of LPR*VEC columns; a wavefront holds G = 64 / LPR lane groups.
//   rows kernel   - one lane group per row (short rows: first-block-column and
//                   diagonal-block entries of the body rows, short head rows)
//   chunks kernel - one wavefront per chunk of a long row (the head rows); the
//                   G lane groups take entries round-robin and are combined
//                   with wavefront shuffles
//   reduce kernel - sums the partial vectors of rows that were split into
//                   several chunks, in a fixed order, and scatters to Y
//   window kernel - diagonal-block tiles with their window of P_i X staged in LDS
//   gather kernel - rows of P_i X materialised (the staged head X_0, or a whole level)
//   panel kernels - optional: head-block entries of sparse head rows with the rows'
//                   accumulators in LDS, one column class per accelerator die
//   corner kernels - the dense top-left corner of the head block in tiles of 256 x 256: the
//                   tile's staged head rows and the row panel's accumulators both live in LDS
//   sddmm kernels - the sampled dense-dense product S = A .* (U V^T) over the same lists
// Both product kernels fetch their entries with coalesced loads into LDS (the
// rows kernel all entries of a workgroup's items at once, the chunk kernel 64
// at a time into a wavefront-private strip, the next 64 already on their way)
// and read them back per lane group, so that U row loads are in flight before
// the first FMA and a lane group only ever waits for the rows it gathers; the
// SIMDs are 16 lanes wide (4 cycles per wavefront instruction), so the inner
// loops are written to need one address instruction per row load.
// Rows written or read exactly once per product (results, partial vectors)
// carry the non-temporal hint and leave the L2 to the rows of X.
// No floating-point atomics: results are bitwise reproducible run to run.
#include <hip/hip_runtime.h>

#include <climits>
#include <cstdint>
#include <type_traits>

#include "arrow_internal.h"
#include "kernel_common.h"

namespace arrow {
namespace {

// ---------------------------------------------------------------------------
// rows kernel: lane group per item of the group list.  A workgroup owns kItemsPerGroupBlock
// consecutive list slots whatever its lane-group width (the die queues of the list rely on it);
// its lane groups take them round-robin.  Entries [lo, mid) of an item read rows of the staged
// head buffer Xh, entries [mid, hi) read rows of X.
// ---------------------------------------------------------------------------
// The workgroup first copies the descriptors of its items and, when they fit the staging buffer
// (they always do for the short rows), all their entries -- one contiguous range -- into LDS with
// coalesced loads; after that the only memory latency a lane group waits for is that of the rows
// it gathers.  A workgroup whose entries do not fit streams them per item through a strip.
constexpr int kRowsStage = 1024;   // entries a workgroup stages at once (8 KiB)

template <int VEC, int LPR, int U, bool SMALL>
__global__ __launch_bounds__(kBlock) void rows_kernel(
    const uint32_t* __restrict__ rows_ptr, const uint32_t* __restrict__ rows_mid,
    const int32_t* __restrict__ rows_dst, const Entry* __restrict__ ent, int64_t n_rows,
    const float* __restrict__ X, const float* __restrict__ Xh, float* __restrict__ Y,
    float* __restrict__ partials, int k, int accumulate) {
  using V = typename Vec<VEC>::type;
  constexpr int GPB = kBlock / LPR;             // lane groups per workgroup
  // entries a lane group parks in LDS per batch: four loads per lane, between 8 and 64 entries
  constexpr int SG = 4 * LPR < 8 ? 8 : (4 * LPR > 64 ? 64 : 4 * LPR);
  constexpr int UU = U < SG ? U : SG;
  constexpr int NST = GPB * SG > kRowsStage ? GPB * SG : kRowsStage;   // the buffer doubles as the per-group strips
  __shared__ Entry stage[NST];
  __shared__ uint32_t s_ptr[kItemsPerGroupBlock + 1];
  __shared__ uint32_t s_mid[kItemsPerGroupBlock];
  __shared__ int32_t s_dst[kItemsPerGroupBlock];
  const int tid = threadIdx.x;
  const int l = tid % LPR;
  const int c = l * VEC + blockIdx.y * (LPR * VEC);
  const bool col_ok = c < k;
  const uint32_t row_bytes = 4u * (uint32_t)k;
  const uint32_t col_bytes = col_ok ? 4u * (uint32_t)c : 0u;   // lanes past the last column read column 0
  const int64_t first = (int64_t)blockIdx.x * kItemsPerGroupBlock;
  const int n_it = n_rows - first < kItemsPerGroupBlock ? (int)(n_rows - first) : kItemsPerGroupBlock;
  if (n_it <= 0) return;
  if (tid <= n_it) s_ptr[tid] = rows_ptr[first + tid];
  if (tid < n_it) { s_mid[tid] = rows_mid[first + tid]; s_dst[tid] = rows_dst[first + tid]; }
  __syncthreads();
  const uint32_t e0 = s_ptr[0];
  const uint32_t total = s_ptr[n_it] - e0;
  const bool staged = total <= (uint32_t)NST;
  if (staged) {
    for (uint32_t t = tid; t < total; t += kBlock) stage[t] = ent[e0 + t];
    __syncthreads();
  }
  Entry* grp = stage + (tid / LPR) * SG;        // the group's SG slots when the entries are streamed
  for (int it = tid / LPR; it < n_it; it += GPB) {
    const int32_t dst = s_dst[it];
    if (dst == INT32_MIN) continue;             // padding slot of the die queues
    const uint32_t lo = s_ptr[it];
    const uint32_t mid = s_mid[it];
    const uint32_t hi = s_ptr[it + 1];
    V acc = vzero<VEC>();
    if (staged) {
      const Entry* se = stage + (lo - e0);
      const uint32_t n = hi - lo, ns = mid > lo ? mid - lo : 0u;
      // entries [0, ns) read the staged head buffer, [ns, n) read X
      for (int seg = 0; seg < 2; ++seg) {
        const char* base = reinterpret_cast<const char*>(seg == 0 ? Xh : X);
        const uint32_t j_hi = seg == 0 ? ns : n;
        for (uint32_t j = seg == 0 ? 0u : ns; j < j_hi; j += UU) {
          Entry e[UU];
          V x[UU];
#pragma unroll
          for (int u = 0; u < UU; ++u) e[u] = se[j + u < j_hi ? j + u : j];
#pragma unroll
          for (int u = 0; u < UU; ++u)
            x[u] = (j + u < j_hi) ? load_row<VEC, SMALL>(base, e[u].xrow, row_bytes, col_bytes) : vzero<VEC>();
#pragma unroll
          for (int u = 0; u < UU; ++u) vfma(acc, (j + u < j_hi) ? e[u].val : 0.f, x[u]);
        }
      }
    } else {
      for (uint32_t b0 = lo; b0 < hi; b0 += SG) {
        const uint32_t nb = hi - b0 < (uint32_t)SG ? hi - b0 : (uint32_t)SG;
#pragma unroll
        for (int t = 0; t < SG / LPR; ++t) {
          const uint32_t idx = (uint32_t)(l + t * LPR);
          if (idx < nb) grp[idx] = ent[b0 + idx];
        }
        strip_sync();
        // entries [0, ns) of the batch read the staged head buffer, [ns, nb) read X
        const uint32_t ns = mid > b0 ? (mid - b0 < nb ? mid - b0 : nb) : 0u;
        for (int seg = 0; seg < 2; ++seg) {
          const char* base = reinterpret_cast<const char*>(seg == 0 ? Xh : X);
          const uint32_t j_hi = seg == 0 ? ns : nb;
          for (uint32_t j = seg == 0 ? 0u : ns; j < j_hi; j += UU) {
            Entry e[UU];
            V x[UU];
#pragma unroll
            for (int u = 0; u < UU; ++u) e[u] = grp[(j + u) % SG];
#pragma unroll
            for (int u = 0; u < UU; ++u)
              x[u] = (j + u < j_hi) ? load_row<VEC, SMALL>(base, e[u].xrow, row_bytes, col_bytes) : vzero<VEC>();
#pragma unroll
            for (int u = 0; u < UU; ++u) vfma(acc, (j + u < j_hi) ? e[u].val : 0.f, x[u]);
          }
        }
        strip_sync();
      }
    }
    if (col_ok) {
      if (dst >= 0) {
        float* y = Y + (size_t)dst * (size_t)k + c;
        if (accumulate) vadd(acc, vload_stream<VEC>(y));
        vstore_stream<VEC>(y, acc);
      } else {
        vstore_stream<VEC>(partials + (size_t)(-1 - dst) * (size_t)k + c, acc);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// chunks kernel: wavefront per chunk.  Entries [lo, mid) of a chunk read rows of the staged
// head buffer Xh, entries [mid, hi) read rows of X (the chunk's entries are ordered by
// column position, head columns first), so the base pointer is uniform inside a batch.
// ---------------------------------------------------------------------------
template <int VEC, int LPR, int U, bool SMALL>
__global__ __launch_bounds__(kBlock) void chunks_kernel(
    const uint32_t* __restrict__ chunk_ptr, const uint32_t* __restrict__ chunk_mid,
    const int32_t* __restrict__ chunk_dst, const Entry* __restrict__ ent, int64_t n_chunks,
    const float* __restrict__ X, const float* __restrict__ Xh, float* __restrict__ Y,
    float* __restrict__ partials, int k, int accumulate) {
  using V = typename Vec<VEC>::type;
  constexpr int G = 64 / LPR;
  constexpr int WPB = kBlock / 64;
  __shared__ Entry strip[WPB][64];
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / 64));
  const int64_t ch = (int64_t)blockIdx.x * WPB + wave;
  if (ch >= n_chunks) return;          // whole wavefront leaves together
  const uint32_t lo = chunk_ptr[ch];
  const uint32_t hi = chunk_ptr[ch + 1];
  if (lo == hi) return;                // padding slot of the die queues
  const uint32_t mid = chunk_mid[ch];
  const int lane = threadIdx.x % 64;
  const int g = lane / LPR;
  const int c = (lane % LPR) * VEC + blockIdx.y * (LPR * VEC);
  const bool col_ok = c < k;
  const uint32_t row_bytes = 4u * (uint32_t)k;
  const uint32_t col_bytes = col_ok ? 4u * (uint32_t)c : 0u;   // lanes past the last column read column 0
  Entry* mine = strip[wave];
  const Entry* grp = mine + g;
  V acc = vzero<VEC>();
  // the next 64 entries of the chunk are fetched while the current batch is being worked on (the
  // two segments are consecutive in the entry array, so the fetch runs across their boundary)
  Entry ahead = ent[lo + lane < hi ? lo + lane : lo];
  for (int seg = 0; seg < 2; ++seg) {
    const char* base = reinterpret_cast<const char*>(seg == 0 ? Xh : X);
    const uint32_t s_lo = seg == 0 ? lo : mid;
    const uint32_t s_hi = seg == 0 ? mid : hi;
    for (uint32_t b0 = s_lo; b0 < s_hi; b0 += 64) {
      const uint32_t nb = s_hi - b0 < 64u ? s_hi - b0 : 64u;
      mine[lane] = ahead;              // entries b0 .. b0 + 63 (those past the chunk's end are not used)
      {
        const uint32_t nx = b0 + nb + lane;     // first entry of the next batch, of this or the next segment
        ahead = ent[nx < hi ? nx : lo];
      }
      strip_sync();
      uint32_t s = 0;                  // step: lane group g handles entry s * G + g
      for (; (s + U) * G <= nb; s += U) {
        Entry e[U];
        V x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) e[u] = grp[(s + u) * G];
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = load_row<VEC, SMALL>(base, e[u].xrow, row_bytes, col_bytes);
#pragma unroll
        for (int u = 0; u < U; ++u) vfma(acc, e[u].val, x[u]);
      }
      if (s * G < nb) {                // last, partly filled round of this batch
        Entry e[U];
        V x[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          ok[u] = (s + u) * G + g < nb;
          e[u] = mine[((s + u) * G + g) % 64];
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
          x[u] = ok[u] ? load_row<VEC, SMALL>(base, e[u].xrow, row_bytes, col_bytes) : vzero<VEC>();
#pragma unroll
        for (int u = 0; u < U; ++u) vfma(acc, ok[u] ? e[u].val : 0.f, x[u]);
      }
      strip_sync();                    // the strip is rewritten by the next batch
    }
  }
  // combine the G lane groups: butterfly over lane-id bits LPR, 2 LPR, ..., 32
#pragma unroll
  for (int m = LPR; m < 64; m <<= 1) vadd(acc, vshfl_xor(acc, m));
  if (g == 0 && col_ok) {
    const int32_t dst = chunk_dst[ch];
    if (dst >= 0) {
      float* y = Y + (size_t)dst * (size_t)k + c;
      if (accumulate) vadd(acc, vload_stream<VEC>(y));
      vstore_stream<VEC>(y, acc);
    } else {
      vstore_stream<VEC>(partials + (size_t)(-1 - dst) * (size_t)k + c, acc);
    }
  }
}

// ---------------------------------------------------------------------------
// window kernel: one workgroup per tile of a diagonal block.  The tile's window of P_i X
// (win_count consecutive positions of the level, one column slice of width LPR * VEC) is
// gathered through perm into LDS once -- the permutation gather of these rows happens here --
// and every diagonal-block entry of the tile's rows then reads its X row from LDS; the rows'
// first-block-column entries read X_0 rows from memory.  One lane group per row.
// ---------------------------------------------------------------------------
constexpr int kWinBlock = 1024;   // threads of a window-kernel workgroup: 16 wavefronts share one staged window

template <int VEC, int LPR>
__global__ __launch_bounds__(kWinBlock) void window_kernel(
    const WindowTile* __restrict__ tiles, const uint32_t* __restrict__ wrow_ptr,
    const uint32_t* __restrict__ wrow_mid, const int32_t* __restrict__ wrow_y,
    const Entry* __restrict__ ent, const int32_t* __restrict__ perm, const float* __restrict__ X,
    float* __restrict__ Y, int k, int accumulate) {
  using V = typename Vec<VEC>::type;
  constexpr int GPB = kWinBlock / LPR;
  constexpr int W = LPR * VEC;                       // columns per slice = LDS row length
  extern __shared__ float win[];                     // win_count x W floats
  const WindowTile t = tiles[blockIdx.x];
  const int l = threadIdx.x % LPR;
  const int grp = threadIdx.x / LPR;
  const int c = l * VEC + blockIdx.y * W;
  const bool col_ok = c < k;
  const float* Xc = X + (col_ok ? c : 0);
  // stage: lane group j loads window rows j, j + GPB, ... four at a time
  for (uint32_t i0 = grp; i0 < t.win_count; i0 += 4 * GPB) {
    int32_t src[4];
    V v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t i = i0 + u * GPB;
      src[u] = i < t.win_count ? perm[t.win_begin + i] : -1;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      v[u] = (src[u] >= 0 && col_ok) ? vload<VEC>(Xc + (size_t)src[u] * (size_t)k) : vzero<VEC>();
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t i = i0 + u * GPB;
      if (i < t.win_count) vstore<VEC>(win + (size_t)i * W + l * VEC, v[u]);
    }
  }
  __syncthreads();
  for (uint32_t wr = t.row_begin + grp; wr < t.row_end; wr += GPB) {
    const uint32_t lo = wrow_ptr[wr], mid = wrow_mid[wr], hi = wrow_ptr[wr + 1];
    V acc = vzero<VEC>();
    for (uint32_t j = lo; j < mid; j += 4) {         // first block column: X_0 rows from memory
      Entry e[4];
      V x[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) e[u] = ent[j + u < mid ? j + u : lo];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        x[u] = (j + u < mid) ? vload<VEC>(Xc + (size_t)e[u].xrow * (size_t)k) : vzero<VEC>();
#pragma unroll
      for (int u = 0; u < 4; ++u) vfma(acc, (j + u < mid) ? e[u].val : 0.f, x[u]);
    }
    for (uint32_t j = mid; j < hi; j += 4) {         // diagonal block: rows of the LDS window
      Entry e[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) e[u] = ent[j + u < hi ? j + u : mid];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (j + u < hi) vfma(acc, e[u].val, vload<VEC>(win + (size_t)e[u].xrow * W + l * VEC));
    }
    if (col_ok) {
      float* y = Y + (size_t)wrow_y[wr] * (size_t)k + c;
      if (accumulate) vadd(acc, vload_stream<VEC>(y));
      vstore_stream<VEC>(y, acc);
    }
  }
}

// ---------------------------------------------------------------------------
// Sampled dense-dense product on the arrow layout:
//     S[src(e)] = a_e * <U[i, :], V[j, :]>       for every stored entry e = (i, j).
// It walks the same work lists as the product kernels.  Per entry the LPR lanes of a group hold
// partial dot products of their VEC columns; NB entries are reduced together by a transposing
// butterfly (each exchange halves the number of live values per lane), so an entry costs about
// one cross-lane exchange instead of log2(LPR).  After the reduction lane l of the group holds the
// dot product of entry l / (LPR / NB) of the batch.  All k columns are covered inside the kernel
// (a loop over column slices of LPR * VEC), so the result needs no second pass.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float vdot(float u, float x) { return u * x; }
__device__ __forceinline__ float vdot(float2 u, float2 x) { return fmaf(u.y, x.y, u.x * x.x); }
__device__ __forceinline__ float vdot(float4 u, float4 x) {
  return fmaf(u.w, x.w, fmaf(u.z, x.z, fmaf(u.y, x.y, u.x * x.x)));
}

template <int NB, int LPR>
__device__ __forceinline__ float group_reduce(float (&p)[NB], int l) {
  int m = LPR / 2;
#pragma unroll
  for (int n = NB; n > 1; n >>= 1) {
    const int half = n / 2;
    const bool upper = (l & m) != 0;          // upper lanes keep the upper half of the entries
#pragma unroll
    for (int e = 0; e < half; ++e) {
      const float send = upper ? p[e] : p[e + half];
      const float keep = upper ? p[e + half] : p[e];
      p[e] = keep + __shfl_xor(send, m, 64);
    }
    m >>= 1;
  }
#pragma unroll
  for (; m >= 1; m >>= 1) p[0] += __shfl_xor(p[0], m, 64);
  return p[0];
}

// Lane group per item of a group list (MODE 0: entries before `mid` read the staged head rows
// Vh, the rest rows of V) or per row of the window-row list (MODE 1: entries before `mid` name
// rows of V, the rest positions inside the row's tile window, translated through perm).
template <int VEC, int LPR, int NB, bool SMALL, int MODE>
__global__ __launch_bounds__(kBlock) void sddmm_rows_kernel(
    const uint32_t* __restrict__ item_ptr, const uint32_t* __restrict__ item_mid,
    const int32_t* __restrict__ item_row, const uint32_t* __restrict__ item_win,
    const int32_t* __restrict__ perm, const Entry* __restrict__ ent,
    const uint32_t* __restrict__ emap, int64_t n_items, const float* __restrict__ U,
    const float* __restrict__ Vm, const float* __restrict__ Vh, float* __restrict__ S, int k,
    int slices) {
  using V = typename Vec<VEC>::type;
  constexpr int GPB = kBlock / LPR;
  constexpr int SG = 4 * LPR < 8 ? 8 : (4 * LPR > 64 ? 64 : 4 * LPR);
  constexpr int W = LPR * VEC;
  constexpr int SPAN = LPR / NB;                 // lanes that end up with the same entry's sum
  __shared__ Entry strip[GPB * SG];
  const int tid = threadIdx.x;
  const int l = tid % LPR;
  const uint32_t row_bytes = 4u * (uint32_t)k;
  Entry* grp = strip + (tid / LPR) * SG;
  const int64_t first = (int64_t)blockIdx.x * kItemsPerGroupBlock;
  for (int it = tid / LPR; it < kItemsPerGroupBlock; it += GPB) {
    const int64_t r = first + it;
    if (r >= n_items) break;
    const int32_t row = item_row[r];
    if (row < 0) continue;                       // padding slot of the die queues
    const uint32_t lo = item_ptr[r];
    const uint32_t mid = item_mid[r];
    const uint32_t hi = item_ptr[r + 1];
    const uint32_t win = MODE == 1 ? item_win[r] : 0u;
    const float* Urow = U + (size_t)row * (size_t)k;
    const V u0 = l * VEC < k ? vload<VEC>(Urow + l * VEC) : vzero<VEC>();
    for (uint32_t b0 = lo; b0 < hi; b0 += SG) {
      const uint32_t nb = hi - b0 < (uint32_t)SG ? hi - b0 : (uint32_t)SG;
#pragma unroll
      for (int t = 0; t < SG / LPR; ++t) {
        const uint32_t idx = (uint32_t)(l + t * LPR);
        if (idx < nb) {
          Entry e = ent[b0 + idx];
          if (MODE == 1 && b0 + idx >= mid) e.xrow = perm[win + (uint32_t)e.xrow];
          grp[idx] = e;
        }
      }
      strip_sync();
      const uint32_t ns = MODE == 1 ? 0u : (mid > b0 ? (mid - b0 < nb ? mid - b0 : nb) : 0u);
      for (int seg = 0; seg < 2; ++seg) {
        const char* base = reinterpret_cast<const char*>(seg == 0 ? Vh : Vm);
        const uint32_t j_hi = seg == 0 ? ns : nb;
        for (uint32_t j = seg == 0 ? 0u : ns; j < j_hi; j += NB) {
          int32_t xr[NB];
          float p[NB];
#pragma unroll
          for (int u = 0; u < NB; ++u) { xr[u] = grp[(j + u) % SG].xrow; p[u] = 0.f; }
          for (int sl = 0; sl < slices; ++sl) {
            const int c = l * VEC + sl * W;
            const bool col_ok = c < k;
            const uint32_t col_bytes = col_ok ? 4u * (uint32_t)c : 0u;
            const V uu = sl == 0 ? u0 : (col_ok ? vload<VEC>(Urow + c) : vzero<VEC>());
            V x[NB];
#pragma unroll
            for (int u = 0; u < NB; ++u)
              x[u] = (j + u < j_hi && col_ok) ? load_row<VEC, SMALL>(base, xr[u], row_bytes, col_bytes)
                                              : vzero<VEC>();
#pragma unroll
            for (int u = 0; u < NB; ++u) p[u] += vdot(uu, x[u]);
          }
          const float dot = group_reduce<NB, LPR>(p, l);
          const uint32_t mine = j + (uint32_t)(l / SPAN);
          if (l % SPAN == 0 && mine < j_hi) S[emap ? emap[b0 + mine] : b0 + mine] = grp[mine % SG].val * dot;
        }
      }
      strip_sync();
    }
  }
}

// Wavefront per item of a wave list: the G lane groups take the item's entries round-robin, NB
// rounds at a time; nothing is combined across lane groups.
template <int VEC, int LPR, int NB, bool SMALL>
__global__ __launch_bounds__(kBlock) void sddmm_chunks_kernel(
    const uint32_t* __restrict__ chunk_ptr, const uint32_t* __restrict__ chunk_mid,
    const int32_t* __restrict__ chunk_row, const Entry* __restrict__ ent,
    const uint32_t* __restrict__ emap, int64_t n_chunks, const float* __restrict__ U,
    const float* __restrict__ Vm, const float* __restrict__ Vh, float* __restrict__ S, int k,
    int slices) {
  using V = typename Vec<VEC>::type;
  constexpr int G = 64 / LPR;
  constexpr int WPB = kBlock / 64;
  constexpr int W = LPR * VEC;
  constexpr int SPAN = LPR / NB;
  __shared__ Entry strip[WPB][64];
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / 64));
  const int64_t ch = (int64_t)blockIdx.x * WPB + wave;
  if (ch >= n_chunks) return;
  const uint32_t lo = chunk_ptr[ch];
  const uint32_t hi = chunk_ptr[ch + 1];
  if (lo == hi) return;                          // padding slot of the die queues
  const uint32_t mid = chunk_mid[ch];
  const int32_t row = chunk_row[ch];
  const int lane = threadIdx.x % 64;
  const int g = lane / LPR;
  const int l = lane % LPR;
  const uint32_t row_bytes = 4u * (uint32_t)k;
  const float* Urow = U + (size_t)row * (size_t)k;
  const V u0 = l * VEC < k ? vload<VEC>(Urow + l * VEC) : vzero<VEC>();
  Entry* mine = strip[wave];
  for (int seg = 0; seg < 2; ++seg) {
    const char* base = reinterpret_cast<const char*>(seg == 0 ? Vh : Vm);
    const uint32_t s_lo = seg == 0 ? lo : mid;
    const uint32_t s_hi = seg == 0 ? mid : hi;
    for (uint32_t b0 = s_lo; b0 < s_hi; b0 += 64) {
      const uint32_t nb = s_hi - b0 < 64u ? s_hi - b0 : 64u;
      if ((uint32_t)lane < nb) mine[lane] = ent[b0 + lane];
      strip_sync();
      for (uint32_t s = 0; s * G < nb; s += NB) {   // round s + u: lane group g handles entry (s + u) * G + g
        int32_t xr[NB];
        float p[NB];
        bool ok[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          const uint32_t idx = (s + u) * G + g;
          ok[u] = idx < nb;
          xr[u] = mine[idx % 64].xrow;
          p[u] = 0.f;
        }
        for (int sl = 0; sl < slices; ++sl) {
          const int c = l * VEC + sl * W;
          const bool col_ok = c < k;
          const uint32_t col_bytes = col_ok ? 4u * (uint32_t)c : 0u;
          const V uu = sl == 0 ? u0 : (col_ok ? vload<VEC>(Urow + c) : vzero<VEC>());
          V x[NB];
#pragma unroll
          for (int u = 0; u < NB; ++u)
            x[u] = (ok[u] && col_ok) ? load_row<VEC, SMALL>(base, xr[u], row_bytes, col_bytes) : vzero<VEC>();
#pragma unroll
          for (int u = 0; u < NB; ++u) p[u] += vdot(uu, x[u]);
        }
        const float dot = group_reduce<NB, LPR>(p, l);
        const uint32_t idx = (s + (uint32_t)(l / SPAN)) * G + g;
        if (l % SPAN == 0 && idx < nb) S[emap ? emap[b0 + idx] : b0 + idx] = mine[idx].val * dot;
      }
      strip_sync();
    }
  }
}

// ---------------------------------------------------------------------------
// panel kernel: workgroup w = group * 8 + class keeps the accumulators of the group's kPanelRows
// head rows (one column slice of LPR * VEC columns) in LDS and runs on accelerator die w mod 8, so
// its entries -- those of the group whose staged head row is of that class -- only touch the
// die's eighth of the staged head.  Each of its kPanelBins lane groups streams one entry list,
// ordered by column window, then row: products are summed in registers while the row stays the
// same and added to the row's LDS accumulator when it changes (all class entries of a row are in
// one stream, so only one lane group ever touches an accumulator and no barrier is needed while
// streaming).  At the end the accumulators go to part[class][slot]; the combine kernel adds the
// eight class results of a row to Y in class order.
// ---------------------------------------------------------------------------
template <int VEC, int LPR, int U, bool SMALL>
__global__ __launch_bounds__(kPanelBins * LPR) void panel_kernel(
    const uint32_t* __restrict__ panel_ptr, const int32_t* __restrict__ panel_y,
    const Entry* __restrict__ ent, int64_t n_bins, int64_t n_slots, const float* __restrict__ Xh,
    float* __restrict__ part, int k) {
  using V = typename Vec<VEC>::type;
  constexpr int W = LPR * VEC;
  constexpr uint32_t kRowMask = (1u << kPanelRowShift) - 1u;
  constexpr int SG = 4 * LPR < 8 ? 8 : (4 * LPR > 32 ? 32 : 4 * LPR);
  constexpr int UU = U < SG ? U : SG;
  constexpr uint32_t kNone = 0xffffffffu;
  __shared__ __attribute__((aligned(16))) float acc[kPanelRows * W];
  __shared__ Entry strip[kPanelBins * SG];
  const int tid = threadIdx.x;
  const int l = tid % LPR;
  const int g = tid / LPR;
  const int c = l * VEC + blockIdx.y * W;
  const bool col_ok = c < k;
  const uint32_t row_bytes = 4u * (uint32_t)k;
  const uint32_t col_bytes = col_ok ? 4u * (uint32_t)c : 0u;
  for (int i = tid; i < kPanelRows * LPR; i += kPanelBins * LPR) vstore<VEC>(acc + i * VEC, vzero<VEC>());
  __syncthreads();
  const int64_t bin = (int64_t)blockIdx.x * kPanelBins + g;
  if (bin < n_bins) {
    const uint32_t lo = panel_ptr[bin], hi = panel_ptr[bin + 1];
    const char* base = reinterpret_cast<const char*>(Xh);
    Entry* grp = strip + g * SG;
    uint32_t cur = kNone;
    V a = vzero<VEC>();
    auto flush_to = [&](uint32_t r) {               // add the register sum to its accumulator, start row r
      if (cur != kNone) {
        float* ap = acc + cur * W + l * VEC;
        V t = vload<VEC>(ap);
        vadd(t, a);
        vstore<VEC>(ap, t);
      }
      cur = r;
      a = vzero<VEC>();
    };
    for (uint32_t b0 = lo; b0 < hi; b0 += SG) {
      const uint32_t nb = hi - b0 < (uint32_t)SG ? hi - b0 : (uint32_t)SG;
#pragma unroll
      for (int t = 0; t < SG / LPR; ++t) {
        const uint32_t idx = (uint32_t)(l + t * LPR);
        if (idx < nb) grp[idx] = ent[b0 + idx];
      }
      strip_sync();
      uint32_t j = 0;
      for (; j + UU <= nb; j += UU) {               // full rounds: nothing is predicated
        Entry e[UU];
        V x[UU];
#pragma unroll
        for (int u = 0; u < UU; ++u) e[u] = grp[j + u];
#pragma unroll
        for (int u = 0; u < UU; ++u)
          x[u] = load_row<VEC, SMALL>(base, (int32_t)((uint32_t)e[u].xrow & kRowMask), row_bytes, col_bytes);
        const uint32_t r0 = (uint32_t)e[0].xrow >> kPanelRowShift;
        const uint32_t r1 = (uint32_t)e[UU - 1].xrow >> kPanelRowShift;
        if (r0 == r1) {                             // the stream is ordered by row: the whole round is one row
          if (r0 != cur) flush_to(r0);
#pragma unroll
          for (int u = 0; u < UU; ++u) vfma(a, e[u].val, x[u]);
        } else {
#pragma unroll
          for (int u = 0; u < UU; ++u) {
            const uint32_t r = (uint32_t)e[u].xrow >> kPanelRowShift;
            if (r != cur) flush_to(r);
            vfma(a, e[u].val, x[u]);
          }
        }
      }
      for (; j < nb; ++j) {                         // the last, partly filled round of the stream
        const Entry e = grp[j];
        const V x = load_row<VEC, SMALL>(base, (int32_t)((uint32_t)e.xrow & kRowMask), row_bytes, col_bytes);
        const uint32_t r = (uint32_t)e.xrow >> kPanelRowShift;
        if (r != cur) flush_to(r);
        vfma(a, e.val, x);
      }
      strip_sync();
    }
    flush_to(kNone);
  }
  __syncthreads();
  const int64_t slot0 = (int64_t)(blockIdx.x / kDies) * kPanelRows;
  const int32_t* py = panel_y + slot0;
  float* out = part + ((size_t)(blockIdx.x % kDies) * (size_t)n_slots + (size_t)slot0) * (size_t)k;
  for (int r = g; r < kPanelRows; r += kPanelBins) {
    if (py[r] < 0 || !col_ok) continue;
    vstore<VEC>(out + (size_t)r * (size_t)k + c, vload<VEC>(acc + r * W + l * VEC));
  }
}

// Y[panel_y[slot]] += part[0][slot] + ... + part[7][slot], lane group per slot.
template <int VEC, int LPR>
__global__ __launch_bounds__(kBlock) void panel_combine_kernel(
    const int32_t* __restrict__ panel_y, int64_t n_slots, const float* __restrict__ part,
    float* __restrict__ Y, int k) {
  using V = typename Vec<VEC>::type;
  constexpr int GPB = kBlock / LPR;
  const int64_t slot = (int64_t)blockIdx.x * GPB + threadIdx.x / LPR;
  const int c = (threadIdx.x % LPR) * VEC + blockIdx.y * (LPR * VEC);
  if (slot >= n_slots || c >= k) return;
  const int32_t y = panel_y[slot];
  if (y < 0) return;
  V p[kDies];
#pragma unroll
  for (int x = 0; x < kDies; ++x)
    p[x] = vload<VEC>(part + ((size_t)x * (size_t)n_slots + (size_t)slot) * (size_t)k + c);
  V acc = p[0];
#pragma unroll
  for (int x = 1; x < kDies; ++x) vadd(acc, p[x]);
  float* yp = Y + (size_t)y * (size_t)k + c;
  vadd(acc, vload<VEC>(yp));
  vstore_stream<VEC>(yp, acc);
}

// Sampled product over the panel entries: lane group per bin, NB entries at a time; the row
// vertex of an entry is looked up through the accumulator table.
template <int VEC, int LPR, int NB, bool SMALL>
__global__ __launch_bounds__(kBlock) void sddmm_panel_kernel(
    const uint32_t* __restrict__ panel_ptr, const int32_t* __restrict__ panel_y,
    const Entry* __restrict__ ent, const uint32_t* __restrict__ emap, int64_t n_bins,
    const float* __restrict__ U, const float* __restrict__ Vh, float* __restrict__ S, int k,
    int slices) {
  using V = typename Vec<VEC>::type;
  constexpr int GPB = kBlock / LPR;
  constexpr int W = LPR * VEC;
  constexpr int SPAN = LPR / NB;
  constexpr uint32_t kRowMask = (1u << kPanelRowShift) - 1u;
  const int l = threadIdx.x % LPR;
  const int64_t bin = (int64_t)blockIdx.x * GPB + threadIdx.x / LPR;
  if (bin >= n_bins) return;
  const uint32_t lo = panel_ptr[bin], hi = panel_ptr[bin + 1];
  const int32_t* py = panel_y + (bin / (kDies * kPanelBins)) * kPanelRows;
  const uint32_t row_bytes = 4u * (uint32_t)k;
  const char* base = reinterpret_cast<const char*>(Vh);
  for (uint32_t j = lo; j < hi; j += NB) {
    int32_t xr[NB], ur[NB];
    float p[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const uint32_t code = (uint32_t)ent[j + u < hi ? j + u : lo].xrow;
      xr[u] = (int32_t)(code & kRowMask);
      ur[u] = py[code >> kPanelRowShift];
      p[u] = 0.f;
    }
    for (int sl = 0; sl < slices; ++sl) {
      const int c = l * VEC + sl * W;
      const bool col_ok = c < k;
      const uint32_t col_bytes = col_ok ? 4u * (uint32_t)c : 0u;
      V x[NB], uu[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const bool ok = j + u < hi && col_ok;
        x[u] = ok ? load_row<VEC, SMALL>(base, xr[u], row_bytes, col_bytes) : vzero<VEC>();
        uu[u] = ok ? vload<VEC>(U + (size_t)ur[u] * (size_t)k + c) : vzero<VEC>();
      }
#pragma unroll
      for (int u = 0; u < NB; ++u) p[u] += vdot(uu[u], x[u]);
    }
    const float dot = group_reduce<NB, LPR>(p, l);
    const uint32_t mine = j + (uint32_t)(l / SPAN);
    if (l % SPAN == 0 && mine < hi) S[emap ? emap[mine] : mine] = ent[mine].val * dot;
  }
}

// ---------------------------------------------------------------------------
// corner kernel: workgroup = one work item = a run of tiles of one row panel (kCornerTile head rows)
// of the dense corner.  The panel's accumulators (one column slice of W = LPR * VEC columns) stay
// in LDS for the whole item.  Per tile the kCornerTile staged head rows it covers are copied into
// LDS with coalesced loads (the next tile's rows are already on their way while the current tile
// is worked on), then every lane group streams one run of the tile's entries: an entry costs one
// LDS row read instead of a row gathered through the caches, and products are summed in registers
// while the row stays the same.  Runs never share a row, so an accumulator has one owner per tile
// and the workgroup barriers between tiles order the owners: no atomics, a fixed summation order.
// Results go to part[item]; the combine kernel adds the items of a panel to Y in item order.
// (A form with one wavefront per run, its 64 lanes across the slice and every entry broadcast
// from a lane so that row changes are scalar branches, was measured at 2.8 ms against 1.8 ms for
// this one on the same 60 M entries.)
// ---------------------------------------------------------------------------
constexpr int kCornerBlock = 1024;

template <int VEC, int LPR, int U>
__global__ __launch_bounds__(kCornerBlock) void corner_kernel(
    const uint32_t* __restrict__ tiles, const uint32_t* __restrict__ items,
    const Entry* __restrict__ ent, const float* __restrict__ Xh, float* __restrict__ part, int k) {
  using V = typename Vec<VEC>::type;
  constexpr int W = LPR * VEC;
  constexpr int GPB = kCornerBlock / LPR;
  constexpr int SG = 4 * LPR < 8 ? 8 : (4 * LPR > 32 ? 32 : 4 * LPR);
  constexpr int UU = U < SG ? U : SG;
  constexpr int NL = (kCornerTile * LPR + kCornerBlock - 1) / kCornerBlock;   // tile elements a thread copies
  constexpr int NA = SG / LPR > 0 ? SG / LPR : 1;     // entries of a batch a lane fetches
  constexpr uint32_t kNone = 0xffffffffu;
  __shared__ __attribute__((aligned(16))) float acc[kCornerTile * W];
  __shared__ __attribute__((aligned(16))) float xt[kCornerTile * W];
  __shared__ Entry strip[GPB * SG];
  const int tid = threadIdx.x;
  const int l = tid % LPR;
  const int g = tid / LPR;
  const int c = l * VEC + blockIdx.y * W;
  const bool col_ok = c < k;
  const uint32_t t_begin = items[blockIdx.x], t_end = items[blockIdx.x + 1];
  for (int i = tid; i < kCornerTile * LPR; i += kCornerBlock) vstore<VEC>(acc + i * VEC, vzero<VEC>());
  // element i of a tile copy: staged row i / LPR, lane slot i % LPR (consecutive threads read
  // consecutive columns of one row)
  V nxt[NL];
  auto fetch = [&](uint32_t t) {
    const uint32_t col0 = tiles[(size_t)t * kCornerTileWords + kCornerRuns + 1];
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      const int i = tid + j * kCornerBlock;
      const int r = i / LPR, cc = (i % LPR) * VEC + blockIdx.y * W;
      nxt[j] = (i < kCornerTile * LPR && cc < k) ? vload<VEC>(Xh + (size_t)(col0 + r) * (size_t)k + cc) : vzero<VEC>();
    }
  };
  fetch(t_begin);
  Entry* grp = strip + g * SG;
  // The first run a lane group takes from a tile, and the first SG entries of that run, are fetched
  // one tile ahead: a run holds about that many entries, so without this every tile would start
  // with two dependent memory latencies (run offsets, then entries) before its first LDS read.
  uint32_t lo_c = 0, hi_c = 0, lo_n = 0, hi_n = 0;
  Entry ahead_c[NA], ahead_n[NA];
  auto fetch_bounds = [&](uint32_t t, uint32_t& lo, uint32_t& hi) {
    lo = hi = 0;
    if (g < kCornerRuns) { lo = tiles[(size_t)t * kCornerTileWords + g]; hi = tiles[(size_t)t * kCornerTileWords + g + 1]; }
  };
  auto fetch_entries = [&](uint32_t lo, uint32_t hi, Entry (&out)[NA]) {
#pragma unroll
    for (int q = 0; q < NA; ++q) {
      const uint32_t idx = lo + (uint32_t)(l + q * LPR);
      out[q] = ent[idx < hi ? idx : (lo < hi ? lo : 0u)];
    }
  };
  fetch_bounds(t_begin, lo_c, hi_c);
  fetch_entries(lo_c, hi_c, ahead_c);
  for (uint32_t t = t_begin; t < t_end; ++t) {
    const bool more = t + 1 < t_end;
    if (more) fetch_bounds(t + 1, lo_n, hi_n);
    __syncthreads();                                  // the previous tile's reads and flushes are done
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      const int i = tid + j * kCornerBlock;
      if (i < kCornerTile * LPR) vstore<VEC>(xt + i * VEC, nxt[j]);
    }
    if (more) fetch(t + 1);
    __syncthreads();
    if (more) fetch_entries(lo_n, hi_n, ahead_n);
    const uint32_t* tw = tiles + (size_t)t * kCornerTileWords;
    for (int run = g; run < kCornerRuns; run += GPB) {
      const bool first = run == g;
      const uint32_t lo = first ? lo_c : tw[run], hi = first ? hi_c : tw[run + 1];
      uint32_t cur = kNone;
      V a = vzero<VEC>();
      auto flush_to = [&](uint32_t r) {               // add the register sum to its accumulator, start row r
        if (cur != kNone) {
          float* ap = acc + cur * W + l * VEC;
          V s = vload<VEC>(ap);
          vadd(s, a);
          vstore<VEC>(ap, s);
        }
        cur = r;
        a = vzero<VEC>();
      };
      for (uint32_t b0 = lo; b0 < hi; b0 += SG) {
        const uint32_t nb = hi - b0 < (uint32_t)SG ? hi - b0 : (uint32_t)SG;
        if (first && b0 == lo) {                      // this batch was fetched while the previous tile ran
#pragma unroll
          for (int q = 0; q < NA; ++q) {
            const uint32_t idx = (uint32_t)(l + q * LPR);
            if (idx < nb) grp[idx] = ahead_c[q];
          }
        } else {
#pragma unroll
          for (int q = 0; q < NA; ++q) {
            const uint32_t idx = (uint32_t)(l + q * LPR);
            if (idx < nb) grp[idx] = ent[b0 + idx];
          }
        }
        strip_sync();
        uint32_t j = 0;
        for (; j + UU <= nb; j += UU) {               // full rounds: nothing is predicated
          Entry e[UU];
          V x[UU];
#pragma unroll
          for (int u = 0; u < UU; ++u) e[u] = grp[j + u];
#pragma unroll
          for (int u = 0; u < UU; ++u) x[u] = vload<VEC>(xt + ((uint32_t)e[u].xrow & 0xffffu) * W + l * VEC);
#pragma unroll
          for (int u = 0; u < UU; ++u) {
            const uint32_t r = (uint32_t)e[u].xrow >> 16;
            if (r != cur) flush_to(r);
            vfma(a, e[u].val, x[u]);
          }
        }
        for (; j < nb; ++j) {                         // the last, partly filled round of the batch
          const Entry e = grp[j];
          const V x = vload<VEC>(xt + ((uint32_t)e.xrow & 0xffffu) * W + l * VEC);
          const uint32_t r = (uint32_t)e.xrow >> 16;
          if (r != cur) flush_to(r);
          vfma(a, e.val, x);
        }
        strip_sync();
      }
      flush_to(kNone);
    }
    lo_c = lo_n; hi_c = hi_n;
#pragma unroll
    for (int q = 0; q < NA; ++q) ahead_c[q] = ahead_n[q];
  }
  __syncthreads();
  float* out = part + (size_t)blockIdx.x * kCornerTile * (size_t)k;
  if (col_ok)
    for (int r = g; r < kCornerTile; r += GPB)
      vstore_stream<VEC>(out + (size_t)r * (size_t)k + c, vload<VEC>(acc + r * W + l * VEC));
}

// Y[corner_y[p]] += part[it][p % kCornerTile] summed over the items it of p's row panel, in item
// order.  Lane group per corner row.
template <int VEC, int LPR>
__global__ __launch_bounds__(kBlock) void corner_combine_kernel(
    const uint32_t* __restrict__ panel_ptr, const int32_t* __restrict__ corner_y, int64_t corner,
    const float* __restrict__ part, float* __restrict__ Y, int k) {
  using V = typename Vec<VEC>::type;
  constexpr int GPB = kBlock / LPR;
  const int64_t p = (int64_t)blockIdx.x * GPB + threadIdx.x / LPR;
  const int c = (threadIdx.x % LPR) * VEC + blockIdx.y * (LPR * VEC);
  if (p >= corner || c >= k) return;
  const uint32_t it0 = panel_ptr[p / kCornerTile], it1 = panel_ptr[p / kCornerTile + 1];
  if (it0 == it1) return;
  const float* src = part + ((size_t)it0 * kCornerTile + (size_t)(p % kCornerTile)) * (size_t)k + c;
  V acc = vload_stream<VEC>(src);
  for (uint32_t it = it0 + 1; it < it1; ++it) {
    src += (size_t)kCornerTile * (size_t)k;
    vadd(acc, vload_stream<VEC>(src));
  }
  float* yp = Y + (size_t)corner_y[p] * (size_t)k + c;
  vadd(acc, vload_stream<VEC>(yp));
  vstore_stream<VEC>(yp, acc);
}

// Sampled product over the corner tiles: workgroup per tile, lane group per run, NB entries at a
// time; the row vertex of an entry comes from the corner row table, its V row from the staged head.
template <int VEC, int LPR, int NB, bool SMALL>
__global__ __launch_bounds__(kBlock) void sddmm_corner_kernel(
    const uint32_t* __restrict__ tiles, const int32_t* __restrict__ corner_y,
    const Entry* __restrict__ ent, const uint32_t* __restrict__ emap, const float* __restrict__ U,
    const float* __restrict__ Vh, float* __restrict__ S, int k, int slices) {
  using V = typename Vec<VEC>::type;
  constexpr int GPB = kBlock / LPR;
  constexpr int W = LPR * VEC;
  constexpr int SPAN = LPR / NB;
  const int l = threadIdx.x % LPR;
  const uint32_t* tw = tiles + (size_t)blockIdx.x * kCornerTileWords;
  const uint32_t col0 = tw[kCornerRuns + 1];
  const int32_t* py = corner_y + (size_t)tw[kCornerRuns + 2] * kCornerTile;
  const uint32_t row_bytes = 4u * (uint32_t)k;
  const char* base = reinterpret_cast<const char*>(Vh);
  for (int run = threadIdx.x / LPR; run < kCornerRuns; run += GPB) {
    const uint32_t lo = tw[run], hi = tw[run + 1];
    for (uint32_t j = lo; j < hi; j += NB) {
      int32_t xr[NB], ur[NB];
      float p[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const uint32_t code = (uint32_t)ent[j + u < hi ? j + u : lo].xrow;
        xr[u] = (int32_t)(col0 + (code & 0xffffu));
        ur[u] = py[code >> 16];
        p[u] = 0.f;
      }
      for (int sl = 0; sl < slices; ++sl) {
        const int c = l * VEC + sl * W;
        const bool col_ok = c < k;
        const uint32_t col_bytes = col_ok ? 4u * (uint32_t)c : 0u;
        V x[NB], uu[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          const bool ok = j + u < hi && col_ok;
          x[u] = ok ? load_row<VEC, SMALL>(base, xr[u], row_bytes, col_bytes) : vzero<VEC>();
          uu[u] = ok ? vload<VEC>(U + (size_t)ur[u] * (size_t)k + c) : vzero<VEC>();
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) p[u] += vdot(uu[u], x[u]);
      }
      const float dot = group_reduce<NB, LPR>(p, l);
      const uint32_t mine = j + (uint32_t)(l / SPAN);
      if (l % SPAN == 0 && mine < hi) S[emap ? emap[mine] : mine] = ent[mine].val * dot;
    }
  }
}

// One wavefront per split row: its partial vectors (consecutive slots) are
// summed slot-strided by the G lane groups, then combined by the same butterfly.
template <int VEC, int LPR>
__global__ __launch_bounds__(kBlock) void reduce_kernel(
    const uint32_t* __restrict__ split_ptr, const int32_t* __restrict__ split_y, int64_t n_split,
    const float* __restrict__ partials, float* __restrict__ Y, int k, int accumulate) {
  using V = typename Vec<VEC>::type;
  constexpr int G = 64 / LPR;
  constexpr int WPB = kBlock / 64;
  const int64_t row = (int64_t)blockIdx.x * WPB + threadIdx.x / 64;
  if (row >= n_split) return;
  const int lane = threadIdx.x % 64;
  const int g = lane / LPR;
  const int c = (lane % LPR) * VEC + blockIdx.y * (LPR * VEC);
  const bool col_ok = c < k;
  const uint32_t lo = split_ptr[row], hi = split_ptr[row + 1];
  const float* __restrict__ Pc = partials + (col_ok ? c : 0);
  V acc = vzero<VEC>();
  uint32_t s = lo + g;
  for (; s + 3 * G < hi; s += 4 * G) {
    V p0 = vload_stream<VEC>(Pc + (size_t)s * (size_t)k);
    V p1 = vload_stream<VEC>(Pc + (size_t)(s + G) * (size_t)k);
    V p2 = vload_stream<VEC>(Pc + (size_t)(s + 2 * G) * (size_t)k);
    V p3 = vload_stream<VEC>(Pc + (size_t)(s + 3 * G) * (size_t)k);
    vadd(acc, p0); vadd(acc, p1); vadd(acc, p2); vadd(acc, p3);
  }
  for (; s < hi; s += G) vadd(acc, vload_stream<VEC>(Pc + (size_t)s * (size_t)k));
#pragma unroll
  for (int m = LPR; m < 64; m <<= 1) vadd(acc, vshfl_xor(acc, m));
  if (g == 0 && col_ok) {
    float* y = Y + (size_t)split_y[row] * (size_t)k + c;
    if (accumulate) vadd(acc, vload_stream<VEC>(y));
    vstore_stream<VEC>(y, acc);
  }
}

template <int VEC, int LPR>
__global__ __launch_bounds__(kBlock) void gather_kernel(const int32_t* __restrict__ perm,
                                                        int64_t n_i, const float* __restrict__ X,
                                                        float* __restrict__ Xp, int k) {
  constexpr int GPB = kBlock / LPR;
  const int64_t p = (int64_t)blockIdx.x * GPB + threadIdx.x / LPR;
  const int c = (threadIdx.x % LPR) * VEC + blockIdx.y * (LPR * VEC);
  if (p >= n_i || c >= k) return;
  vstore<VEC>(Xp + (size_t)p * (size_t)k + c, vload<VEC>(X + (size_t)perm[p] * (size_t)k + c));
}

}  // namespace

int launch_rows(const uint32_t* rows_ptr, const uint32_t* rows_mid, const int32_t* rows_dst,
                const Entry* entries, int64_t n_rows, const float* X, int64_t x_rows,
                const float* Xh, float* Y, float* partials, int32_t k, bool accumulate,
                const LaunchTuning& t, void* stream) {
  if (n_rows <= 0) return 0;
  const Shape s = pick_shape(k, t.kc);
  const bool small = small_matrix(x_rows, k);
  return dispatch_shape(s, [&](auto V, auto L) -> int {
    constexpr int VEC = decltype(V)::value, LPR = decltype(L)::value;
    // a multiple of 8 workgroups per column slice: workgroup w of every slice runs on die w mod 8
    const int64_t blocks = ceil_div(ceil_div(n_rows, kItemsPerGroupBlock), kDies) * kDies;
    if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)blocks, (unsigned)s.slices);
    if (small)
      hipLaunchKernelGGL((rows_kernel<VEC, LPR, 8, true>), grid, dim3(kBlock), 0, (hipStream_t)stream,
                         rows_ptr, rows_mid, rows_dst, entries, n_rows, X, Xh, Y, partials, (int)k,
                         accumulate ? 1 : 0);
    else
      hipLaunchKernelGGL((rows_kernel<VEC, LPR, 8, false>), grid, dim3(kBlock), 0, (hipStream_t)stream,
                         rows_ptr, rows_mid, rows_dst, entries, n_rows, X, Xh, Y, partials, (int)k,
                         accumulate ? 1 : 0);
    return (int)hipGetLastError();
  });
}

int launch_chunks(const uint32_t* chunk_ptr, const uint32_t* chunk_mid, const int32_t* chunk_dst,
                  const Entry* entries, int64_t n_chunks, const float* X, int64_t x_rows,
                  const float* Xh, float* Y, float* partials, int32_t k, bool accumulate,
                  const LaunchTuning& t, void* stream) {
  if (n_chunks <= 0) return 0;
  const Shape s = pick_shape(k, t.kc);
  const bool small = small_matrix(x_rows, k);    // the staged buffer has at most as many rows as X
  return dispatch_shape(s, [&](auto V, auto L) -> int {
    constexpr int VEC = decltype(V)::value, LPR = decltype(L)::value;
    // a multiple of 8 workgroups per column slice, so that workgroup w of every slice runs on
    // die w mod 8 (the die queues of the chunk list rely on it)
    const int64_t blocks = ceil_div(ceil_div(n_chunks, kBlock / 64), kDies) * kDies;
    if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)blocks, (unsigned)s.slices);
    if (small)
      hipLaunchKernelGGL((chunks_kernel<VEC, LPR, 8, true>), grid, dim3(kBlock), 0, (hipStream_t)stream,
                         chunk_ptr, chunk_mid, chunk_dst, entries, n_chunks, X, Xh, Y, partials,
                         (int)k, accumulate ? 1 : 0);
    else
      hipLaunchKernelGGL((chunks_kernel<VEC, LPR, 8, false>), grid, dim3(kBlock), 0, (hipStream_t)stream,
                         chunk_ptr, chunk_mid, chunk_dst, entries, n_chunks, X, Xh, Y, partials,
                         (int)k, accumulate ? 1 : 0);
    return (int)hipGetLastError();
  });
}

int launch_reduce(const uint32_t* split_ptr, const int32_t* split_y, int64_t n_split,
                  const float* partials, float* Y, int32_t k, bool accumulate, void* stream) {
  if (n_split <= 0) return 0;
  const Shape s = pick_shape(k, 0);
  return dispatch_shape(s, [&](auto V, auto L) -> int {
    constexpr int VEC = decltype(V)::value, LPR = decltype(L)::value;
    const int64_t blocks = ceil_div(n_split, kBlock / 64);
    if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)blocks, (unsigned)s.slices);
    hipLaunchKernelGGL((reduce_kernel<VEC, LPR>), grid, dim3(kBlock), 0, (hipStream_t)stream,
                       split_ptr, split_y, n_split, partials, Y, (int)k, accumulate ? 1 : 0);
    return (int)hipGetLastError();
  });
}

int launch_gather(const int32_t* perm, int64_t n_i, const float* X, float* Xp, int32_t k,
                  void* stream) {
  if (n_i <= 0) return 0;
  const Shape s = pick_shape(k, 0);
  return dispatch_shape(s, [&](auto V, auto L) -> int {
    constexpr int VEC = decltype(V)::value, LPR = decltype(L)::value;
    const int64_t blocks = ceil_div(n_i, kBlock / LPR);
    if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)blocks, (unsigned)s.slices);
    hipLaunchKernelGGL((gather_kernel<VEC, LPR>), grid, dim3(kBlock), 0, (hipStream_t)stream, perm,
                       n_i, X, Xp, (int)k);
    return (int)hipGetLastError();
  });
}

int launch_window(const WindowTile* tiles, int64_t n_tiles, int64_t max_span, const uint32_t* wrow_ptr,
                  const uint32_t* wrow_mid, const int32_t* wrow_y, const Entry* entries,
                  const int32_t* perm, const float* X, float* Y, int32_t k, bool accumulate,
                  void* stream) {
  if (n_tiles <= 0) return 0;
  // widest column slice whose window still fits the 64 KiB of LDS a workgroup may use
  const int64_t lds_budget = 64 * 1024;
  int kc = 256;
  while (kc > 1 && max_span * kc * 4 > lds_budget) kc >>= 1;
  if (max_span * kc * 4 > lds_budget) return (int)hipErrorInvalidValue;
  const Shape s = pick_shape(k, kc);
  if (max_span * (int64_t)(s.lpr * s.vec) * 4 > lds_budget) return (int)hipErrorInvalidValue;
  return dispatch_shape(s, [&](auto V, auto L) -> int {
    constexpr int VEC = decltype(V)::value, LPR = decltype(L)::value;
    if (n_tiles > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)n_tiles, (unsigned)s.slices);
    const size_t lds = (size_t)max_span * LPR * VEC * sizeof(float);
    hipLaunchKernelGGL((window_kernel<VEC, LPR>), grid, dim3(kWinBlock), lds, (hipStream_t)stream, tiles,
                       wrow_ptr, wrow_mid, wrow_y, entries, perm, X, Y, (int)k, accumulate ? 1 : 0);
    return (int)hipGetLastError();
  });
}

namespace {
// entries a lane group reduces together (= row loads in flight per lane); 4 measured best of 4, 8, 16
constexpr int kSddmmBatch = 4;
template <int LPR> struct BatchOf { static constexpr int value = LPR < kSddmmBatch ? LPR : kSddmmBatch; };
}  // namespace

int launch_sddmm_rows(int mode, const uint32_t* item_ptr, const uint32_t* item_mid,
                      const int32_t* item_row, const uint32_t* item_win, const int32_t* perm,
                      const Entry* entries, const uint32_t* emap, int64_t n_items, const float* U,
                      const float* V, int64_t v_rows, const float* Vh, float* S, int32_t k,
                      void* stream) {
  if (n_items <= 0) return 0;
  const Shape s = pick_shape(k, 0);
  const bool small = small_matrix(v_rows, k);
  return dispatch_shape(s, [&](auto Vc, auto L) -> int {
    constexpr int VEC = decltype(Vc)::value, LPR = decltype(L)::value, NB = BatchOf<LPR>::value;
    const int64_t blocks = ceil_div(ceil_div(n_items, kItemsPerGroupBlock), kDies) * kDies;
    if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)blocks);
#define ARROW_LAUNCH(SM, MD)                                                                       \
  hipLaunchKernelGGL((sddmm_rows_kernel<VEC, LPR, NB, SM, MD>), grid, dim3(kBlock), 0,             \
                     (hipStream_t)stream, item_ptr, item_mid, item_row, item_win, perm, entries,   \
                     emap, n_items, U, V, Vh, S, (int)k, (int)s.slices)
    if (mode == 0) { if (small) ARROW_LAUNCH(true, 0); else ARROW_LAUNCH(false, 0); }
    else           { if (small) ARROW_LAUNCH(true, 1); else ARROW_LAUNCH(false, 1); }
#undef ARROW_LAUNCH
    return (int)hipGetLastError();
  });
}

int launch_sddmm_chunks(const uint32_t* chunk_ptr, const uint32_t* chunk_mid, const int32_t* chunk_row,
                        const Entry* entries, const uint32_t* emap, int64_t n_chunks, const float* U,
                        const float* V, int64_t v_rows, const float* Vh, float* S, int32_t k,
                        void* stream) {
  if (n_chunks <= 0) return 0;
  const Shape s = pick_shape(k, 0);
  const bool small = small_matrix(v_rows, k);
  return dispatch_shape(s, [&](auto Vc, auto L) -> int {
    constexpr int VEC = decltype(Vc)::value, LPR = decltype(L)::value, NB = BatchOf<LPR>::value;
    const int64_t blocks = ceil_div(ceil_div(n_chunks, kBlock / 64), kDies) * kDies;
    if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)blocks);
    if (small)
      hipLaunchKernelGGL((sddmm_chunks_kernel<VEC, LPR, NB, true>), grid, dim3(kBlock), 0, (hipStream_t)stream,
                         chunk_ptr, chunk_mid, chunk_row, entries, emap, n_chunks, U, V, Vh, S, (int)k,
                         (int)s.slices);
    else
      hipLaunchKernelGGL((sddmm_chunks_kernel<VEC, LPR, NB, false>), grid, dim3(kBlock), 0, (hipStream_t)stream,
                         chunk_ptr, chunk_mid, chunk_row, entries, emap, n_chunks, U, V, Vh, S, (int)k,
                         (int)s.slices);
    return (int)hipGetLastError();
  });
}

namespace {
// (VEC, LPR) with at most 32 lanes per row: the panel kernel runs kPanelBins lane groups per workgroup
template <typename F>
int dispatch_narrow(const Shape& s, F&& f) {
#define ARROW_CASE(V, L) \
  if (s.vec == V && s.lpr == L) return f(std::integral_constant<int, V>{}, std::integral_constant<int, L>{});
#define ARROW_CASES(V) ARROW_CASE(V, 1) ARROW_CASE(V, 2) ARROW_CASE(V, 4) ARROW_CASE(V, 8) ARROW_CASE(V, 16) ARROW_CASE(V, 32)
  ARROW_CASES(4)
  ARROW_CASES(2)
  ARROW_CASES(1)
#undef ARROW_CASES
#undef ARROW_CASE
  return (int)hipErrorInvalidValue;
}
}  // namespace

int launch_panel(const uint32_t* panel_ptr, const int32_t* panel_y, const Entry* entries,
                 int64_t n_groups, const float* Xh, int64_t xh_rows, float* part, int32_t k, void* stream) {
  if (n_groups <= 0) return 0;
  const int vec = (k % 4 == 0) ? 4 : (k % 2 == 0) ? 2 : 1;
  const Shape s = pick_shape(k, 32 * vec);         // at most 32 lanes per row: LDS rows of at most 128 floats
  const bool small = small_matrix(xh_rows, k);
  return dispatch_narrow(s, [&](auto Vc, auto L) -> int {
    constexpr int VEC = decltype(Vc)::value, LPR = decltype(L)::value;
    const int64_t blocks = n_groups * kDies;          // workgroup id mod 8 = column class = die
    if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    const int64_t n_bins = blocks * kPanelBins, n_slots = n_groups * kPanelRows;
    dim3 grid((unsigned)blocks, (unsigned)s.slices);
    if (small)
      hipLaunchKernelGGL((panel_kernel<VEC, LPR, 8, true>), grid, dim3(kPanelBins * LPR), 0, (hipStream_t)stream,
                         panel_ptr, panel_y, entries, n_bins, n_slots, Xh, part, (int)k);
    else
      hipLaunchKernelGGL((panel_kernel<VEC, LPR, 8, false>), grid, dim3(kPanelBins * LPR), 0, (hipStream_t)stream,
                         panel_ptr, panel_y, entries, n_bins, n_slots, Xh, part, (int)k);
    return (int)hipGetLastError();
  });
}

int launch_panel_combine(const int32_t* panel_y, int64_t n_slots, const float* part, float* Y, int32_t k,
                         void* stream) {
  if (n_slots <= 0) return 0;
  const Shape s = pick_shape(k, 0);
  return dispatch_shape(s, [&](auto Vc, auto L) -> int {
    constexpr int VEC = decltype(Vc)::value, LPR = decltype(L)::value;
    const int64_t blocks = ceil_div(n_slots, kBlock / LPR);
    if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)blocks, (unsigned)s.slices);
    hipLaunchKernelGGL((panel_combine_kernel<VEC, LPR>), grid, dim3(kBlock), 0, (hipStream_t)stream, panel_y,
                       n_slots, part, Y, (int)k);
    return (int)hipGetLastError();
  });
}

int launch_sddmm_panel(const uint32_t* panel_ptr, const int32_t* panel_y, const Entry* entries,
                       const uint32_t* emap, int64_t n_bins, const float* U, const float* Vh,
                       int64_t vh_rows, float* S, int32_t k, void* stream) {
  if (n_bins <= 0) return 0;
  const Shape s = pick_shape(k, 0);
  const bool small = small_matrix(vh_rows, k);
  return dispatch_shape(s, [&](auto Vc, auto L) -> int {
    constexpr int VEC = decltype(Vc)::value, LPR = decltype(L)::value, NB = BatchOf<LPR>::value;
    const int64_t blocks = ceil_div(n_bins, kBlock / LPR);
    if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)blocks);
    if (small)
      hipLaunchKernelGGL((sddmm_panel_kernel<VEC, LPR, NB, true>), grid, dim3(kBlock), 0, (hipStream_t)stream,
                         panel_ptr, panel_y, entries, emap, n_bins, U, Vh, S, (int)k, (int)s.slices);
    else
      hipLaunchKernelGGL((sddmm_panel_kernel<VEC, LPR, NB, false>), grid, dim3(kBlock), 0, (hipStream_t)stream,
                         panel_ptr, panel_y, entries, emap, n_bins, U, Vh, S, (int)k, (int)s.slices);
    return (int)hipGetLastError();
  });
}


namespace {
// (VEC, LPR) with at most 64 columns per slice: the corner kernel keeps 2 x 256 rows of a slice in LDS
template <typename F>
int dispatch_w64(const Shape& s, F&& f) {
#define ARROW_CASE(V, L) \
  if (s.vec == V && s.lpr == L) return f(std::integral_constant<int, V>{}, std::integral_constant<int, L>{});
  ARROW_CASE(4, 1) ARROW_CASE(4, 2) ARROW_CASE(4, 4) ARROW_CASE(4, 8) ARROW_CASE(4, 16)
  ARROW_CASE(2, 1) ARROW_CASE(2, 2) ARROW_CASE(2, 4) ARROW_CASE(2, 8) ARROW_CASE(2, 16) ARROW_CASE(2, 32)
  ARROW_CASE(1, 1) ARROW_CASE(1, 2) ARROW_CASE(1, 4) ARROW_CASE(1, 8) ARROW_CASE(1, 16) ARROW_CASE(1, 32) ARROW_CASE(1, 64)
#undef ARROW_CASE
  return (int)hipErrorInvalidValue;
}
}  // namespace

int launch_corner(const uint32_t* tiles, const uint32_t* items, int64_t n_items, const Entry* entries,
                  const float* Xh, int64_t xh_rows, float* part, int32_t k, void* stream) {
  if (n_items <= 0) return 0;
  (void)xh_rows;
  // 64-column slices: accumulators and tile copy take 64 KiB of LDS each
  const Shape s = pick_shape(k, 64);
  return dispatch_w64(s, [&](auto Vc, auto L) -> int {
    constexpr int VEC = decltype(Vc)::value, LPR = decltype(L)::value;
    if (n_items > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)n_items, (unsigned)s.slices);
    hipLaunchKernelGGL((corner_kernel<VEC, LPR, 8>), grid, dim3(kCornerBlock), 0, (hipStream_t)stream, tiles,
                       items, entries, Xh, part, (int)k);
    return (int)hipGetLastError();
  });
}

int launch_corner_combine(const uint32_t* panel_ptr, const int32_t* corner_y, int64_t corner,
                          const float* part, float* Y, int32_t k, void* stream) {
  if (corner <= 0) return 0;
  const Shape s = pick_shape(k, 0);
  return dispatch_shape(s, [&](auto Vc, auto L) -> int {
    constexpr int VEC = decltype(Vc)::value, LPR = decltype(L)::value;
    const int64_t blocks = ceil_div(corner, kBlock / LPR);
    if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)blocks, (unsigned)s.slices);
    hipLaunchKernelGGL((corner_combine_kernel<VEC, LPR>), grid, dim3(kBlock), 0, (hipStream_t)stream,
                       panel_ptr, corner_y, corner, part, Y, (int)k);
    return (int)hipGetLastError();
  });
}

int launch_sddmm_corner(const uint32_t* tiles, int64_t n_tiles, const int32_t* corner_y, const Entry* entries,
                        const uint32_t* emap, const float* U, const float* Vh, int64_t vh_rows, float* S,
                        int32_t k, void* stream) {
  if (n_tiles <= 0) return 0;
  const Shape s = pick_shape(k, 0);
  const bool small = small_matrix(vh_rows, k);
  return dispatch_shape(s, [&](auto Vc, auto L) -> int {
    constexpr int VEC = decltype(Vc)::value, LPR = decltype(L)::value, NB = BatchOf<LPR>::value;
    if (n_tiles > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)n_tiles);
    if (small)
      hipLaunchKernelGGL((sddmm_corner_kernel<VEC, LPR, NB, true>), grid, dim3(kBlock), 0, (hipStream_t)stream,
                         tiles, corner_y, entries, emap, U, Vh, S, (int)k, (int)s.slices);
    else
      hipLaunchKernelGGL((sddmm_corner_kernel<VEC, LPR, NB, false>), grid, dim3(kBlock), 0, (hipStream_t)stream,
                         tiles, corner_y, entries, emap, U, Vh, S, (int)k, (int)s.slices);
    return (int)hipGetLastError();
  });
}

}  // namespace arrow
