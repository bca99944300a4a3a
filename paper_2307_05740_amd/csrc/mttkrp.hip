// HIP kernel for gfx950 of the order-3 MTTKRP
//     A(i, a) = sum_{j,k} T(i, j, k) B(j, a) C(k, a)
// in the factorize-and-fuse form (the paper's sections "Pairwise Contraction" and "Performance
// Evaluation"): per fibre (i, j) the sum x(a) = sum_k T(i,j,k) C(k,a) is formed first -- the same
// scaled vector update over the dense index as the matrix product's leaf -- and then multiplied
// elementwise by B(j, :) and added to the slice's accumulator, so the intermediate never leaves
// registers and the products with B are paid per fibre, not per entry.
//
// A lane owns VEC consecutive columns of the rank index, LPR lanes cover a slice of LPR * VEC
// columns, a wavefront holds G = 64 / LPR lane groups.  One wavefront per work item (a run of
// segments of one slice i, at most kCsfItemNnz entries and kCsfItemSegs segments, each segment
// being at most 64 entries of one fibre).  The wavefront first copies the item's entries and
// segment descriptors into LDS with coalesced loads; its lane groups then take the segments
// round-robin and read offsets, j and entries from there, so that the only memory latency inside
// the loop is that of the gathered rows (the row of B and up to U rows of C at a time; working on
// two to four segments at once was measured and is no faster).  At the end the lane groups are combined with wavefront shuffles and the
// result goes to row i of A or, for a slice cut into several items, to a partial vector that the
// reduction kernel sums in a fixed order.  No atomics.
#include <hip/hip_runtime.h>

#include <climits>
#include <cstdint>

#include "arrow_internal.h"
#include "kernel_common.h"

namespace arrow {
namespace {

__device__ __forceinline__ void vmuladd(float& a, float x, float b) { a = fmaf(x, b, a); }
__device__ __forceinline__ void vmuladd(float2& a, float2 x, float2 b) {
  a.x = fmaf(x.x, b.x, a.x); a.y = fmaf(x.y, b.y, a.y);
}
__device__ __forceinline__ void vmuladd(float4& a, float4 x, float4 b) {
  a.x = fmaf(x.x, b.x, a.x); a.y = fmaf(x.y, b.y, a.y); a.z = fmaf(x.z, b.z, a.z); a.w = fmaf(x.w, b.w, a.w);
}

template <int VEC, int LPR, int U, bool SMALL_B, bool SMALL_C>
__global__ __launch_bounds__(kBlock) void mttkrp_kernel(
    const uint32_t* __restrict__ item_seg, const uint32_t* __restrict__ item_ent,
    const int32_t* __restrict__ item_dst, const uint32_t* __restrict__ seg_ptr,
    const int32_t* __restrict__ seg_j, const Entry* __restrict__ ent, int64_t n_items,
    const float* __restrict__ B, const float* __restrict__ C, float* __restrict__ A,
    float* __restrict__ partials, int R) {
  using V = typename Vec<VEC>::type;
  constexpr int G = 64 / LPR;
  constexpr int WPB = kBlock / 64;
  __shared__ Entry s_ent[WPB][kCsfItemNnz];
  __shared__ uint32_t s_ptr[WPB][kCsfItemSegs + 1];     // segment offsets relative to the item's first entry
  __shared__ int32_t s_j[WPB][kCsfItemSegs];
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / 64));
  const int64_t it = (int64_t)blockIdx.x * WPB + wave;
  if (it >= n_items) return;            // whole wavefront leaves together
  const uint32_t s_lo = item_seg[it], e_lo = item_ent[it];
  uint32_t n_seg = item_seg[it + 1] - s_lo, n_ent = item_ent[it + 1] - e_lo;
  // An item beyond what the staging arrays hold cannot come out of csf3_build, which is the one
  // place that enforces the limits; if an image ever carried one, its destination row is filled
  // with NaN (a result that announces itself) instead of being left with whatever it held.
  const bool over_limit = n_seg > (uint32_t)kCsfItemSegs || n_ent > (uint32_t)kCsfItemNnz;
  if (over_limit) { n_seg = 0; n_ent = 0; }
  const int lane = threadIdx.x % 64;
  const int g = lane / LPR;
  const int c = (lane % LPR) * VEC + blockIdx.y * (LPR * VEC);
  const bool col_ok = c < R;
  const uint32_t row_bytes = 4u * (uint32_t)R;
  const uint32_t col_bytes = col_ok ? 4u * (uint32_t)c : 0u;   // lanes past the last column read column 0
  const char* Bb = reinterpret_cast<const char*>(B);
  const char* Cb = reinterpret_cast<const char*>(C);
  // stage the item: n_seg <= kCsfItemSegs and n_ent <= kCsfItemNnz by construction of the image
  for (uint32_t t = lane; t <= n_seg; t += 64) s_ptr[wave][t] = seg_ptr[s_lo + t] - e_lo;
  for (uint32_t t = lane; t < n_seg; t += 64) s_j[wave][t] = seg_j[s_lo + t];
  for (uint32_t t = lane; t < n_ent; t += 64) s_ent[wave][t] = ent[e_lo + t];
  strip_sync();
  const Entry* se = s_ent[wave];
  V acc = vzero<VEC>();
  for (uint32_t s = g; s < n_seg; s += G) {
    const uint32_t lo = s_ptr[wave][s], hi = s_ptr[wave][s + 1];
    const V b = load_row<VEC, SMALL_B>(Bb, s_j[wave][s], row_bytes, col_bytes);
    V x = vzero<VEC>();
    for (uint32_t p = lo; p < hi; p += U) {
      Entry e[U];
      V cr[U];
#pragma unroll
      for (int u = 0; u < U; ++u) e[u] = se[p + u < hi ? p + u : lo];
#pragma unroll
      for (int u = 0; u < U; ++u)
        cr[u] = p + u < hi ? load_row<VEC, SMALL_C>(Cb, e[u].xrow, row_bytes, col_bytes) : vzero<VEC>();
#pragma unroll
      for (int u = 0; u < U; ++u) vfma(x, p + u < hi ? e[u].val : 0.f, cr[u]);
    }
    vmuladd(acc, x, b);
  }
#pragma unroll
  for (int m = LPR; m < 64; m <<= 1) vadd(acc, vshfl_xor(acc, m));
  if (over_limit) vfma(acc, __builtin_nanf(""), acc);
  if (g == 0 && col_ok) {
    const int32_t dst = item_dst[it];
    if (dst >= 0) vstore<VEC>(A + (size_t)dst * (size_t)R + c, acc);
    else vstore<VEC>(partials + (size_t)(-1 - dst) * (size_t)R + c, acc);
  }
}

}  // namespace

int launch_mttkrp(const uint32_t* item_seg, const uint32_t* item_ent, const int32_t* item_dst,
                  const uint32_t* seg_ptr, const int32_t* seg_j, const Entry* entries, int64_t n_items, const float* B,
                  int64_t b_rows, const float* C, int64_t c_rows, float* A, float* partials, int32_t R,
                  double mean_segment, void* stream) {
  if (n_items <= 0) return 0;
  // row loads issued per round of a segment: more than the segments hold only adds predicated slots
  const int rounds = mean_segment < 2.5 ? 2 : (mean_segment < 6.0 ? 4 : 8);
  const Shape s = pick_shape(R, 0);
  const bool small_b = small_matrix(b_rows, R), small_c = small_matrix(c_rows, R);
  return dispatch_shape(s, [&](auto Vc, auto L) -> int {
    constexpr int VEC = decltype(Vc)::value, LPR = decltype(L)::value;
    const int64_t blocks = ceil_div(n_items, kBlock / 64);
    if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)blocks, (unsigned)s.slices);
#define ARROW_LAUNCH(UU, SM)                                                                        \
  hipLaunchKernelGGL((mttkrp_kernel<VEC, LPR, UU, SM, SM>), grid, dim3(kBlock), 0, (hipStream_t)stream, \
                     item_seg, item_ent, item_dst, seg_ptr, seg_j, entries, n_items, B, C, A, partials, (int)R)
    if (small_b && small_c) {
      if (rounds == 2) ARROW_LAUNCH(2, true); else if (rounds == 4) ARROW_LAUNCH(4, true); else ARROW_LAUNCH(8, true);
    } else {
      if (rounds == 2) ARROW_LAUNCH(2, false); else if (rounds == 4) ARROW_LAUNCH(4, false); else ARROW_LAUNCH(8, false);
    }
#undef ARROW_LAUNCH
    return (int)hipGetLastError();
  });
}

}  // namespace arrow
