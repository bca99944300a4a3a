// HIP kernels for gfx950 (CDNA4, 64-wide wavefronts) of the arrow SpMM
//     Y = sum_i P_i^T B_i (P_i X).
//
// Every kernel keeps the dense index innermost and contiguous across lanes:
// one stored entry a(p,q) triggers one scaled vector update
//     acc[0:k] += a * X[perm[q], 0:k]
// which is the axpy leaf of the paper's loop nests (figure "Loop nest for an
// order 4 TTMc kernel") at order 2, with rows then nonzeros as outer loops
// (section "SpTTN-Cyclops Framework": sparse indices in stored order).  The
// row gather P_i X is fused into the loads: entries carry perm[q] directly.
// The scatter P_i^T is fused into the epilogue: results go to row perm[p] of Y.
//
// A lane owns VEC consecutive columns; LPR lanes ("a lane group") cover one
// slice of LPR*VEC columns; a wavefront holds G = 64 / LPR lane groups.
//   rows kernel   - one lane group per row (short rows: first-block-column and
//                   diagonal-block entries of the body rows, short head rows)
//   chunks kernel - one wavefront per chunk of <= chunk_nnz entries of a long
//                   row (the head rows); the G lane groups take entries
//                   round-robin and are combined with wavefront shuffles
//   reduce kernel - sums the partial vectors of rows that were split into
//                   several chunks, in a fixed order, and scatters to Y
//   gather kernel - P_i X materialised (not used by the fused path)
// No floating-point atomics: results are bitwise reproducible run to run.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "arrow_internal.h"

namespace arrow {
namespace {

constexpr int kBlock = 256;  // threads per workgroup = 4 wavefronts
constexpr int kXcds = 8;     // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin

template <int VEC> struct Vec;
template <> struct Vec<1> { using type = float; };
template <> struct Vec<2> { using type = float2; };
template <> struct Vec<4> { using type = float4; };

template <int VEC> __device__ __forceinline__ typename Vec<VEC>::type vzero();
template <> __device__ __forceinline__ float vzero<1>() { return 0.f; }
template <> __device__ __forceinline__ float2 vzero<2>() { return make_float2(0.f, 0.f); }
template <> __device__ __forceinline__ float4 vzero<4>() { return make_float4(0.f, 0.f, 0.f, 0.f); }

__device__ __forceinline__ void vfma(float& a, float s, float x) { a = fmaf(s, x, a); }
__device__ __forceinline__ void vfma(float2& a, float s, float2 x) {
  a.x = fmaf(s, x.x, a.x); a.y = fmaf(s, x.y, a.y);
}
__device__ __forceinline__ void vfma(float4& a, float s, float4 x) {
  a.x = fmaf(s, x.x, a.x); a.y = fmaf(s, x.y, a.y); a.z = fmaf(s, x.z, a.z); a.w = fmaf(s, x.w, a.w);
}
__device__ __forceinline__ void vadd(float& a, float x) { a += x; }
__device__ __forceinline__ void vadd(float2& a, float2 x) { a.x += x.x; a.y += x.y; }
__device__ __forceinline__ void vadd(float4& a, float4 x) { a.x += x.x; a.y += x.y; a.z += x.z; a.w += x.w; }

__device__ __forceinline__ float vshfl_xor(float v, int m) { return __shfl_xor(v, m, 64); }
__device__ __forceinline__ float2 vshfl_xor(float2 v, int m) {
  return make_float2(__shfl_xor(v.x, m, 64), __shfl_xor(v.y, m, 64));
}
__device__ __forceinline__ float4 vshfl_xor(float4 v, int m) {
  return make_float4(__shfl_xor(v.x, m, 64), __shfl_xor(v.y, m, 64), __shfl_xor(v.z, m, 64),
                     __shfl_xor(v.w, m, 64));
}

template <int VEC>
__device__ __forceinline__ typename Vec<VEC>::type vload(const float* p) {
  return *reinterpret_cast<const typename Vec<VEC>::type*>(p);
}
template <int VEC>
__device__ __forceinline__ void vstore(float* p, typename Vec<VEC>::type v) {
  *reinterpret_cast<typename Vec<VEC>::type*>(p) = v;
}

// Workgroups are dealt to the 8 dies round-robin; this maps the physical
// workgroup id to a logical one so that each die walks one contiguous eighth
// of the work list (its L2 then sees one neighbourhood of rows / windows).
__device__ __forceinline__ int64_t logical_block(int64_t phys, int64_t per_xcd, int remap) {
  return remap ? (phys % kXcds) * per_xcd + phys / kXcds : phys;
}

template <int VEC, int LPR, int U>
__global__ __launch_bounds__(kBlock) void rows_kernel(
    const uint32_t* __restrict__ rows_ptr, const int32_t* __restrict__ rows_y,
    const Entry* __restrict__ ent, int64_t n_rows, const float* __restrict__ X,
    float* __restrict__ Y, int k, int accumulate, int64_t per_xcd, int remap) {
  using V = typename Vec<VEC>::type;
  constexpr int GPB = kBlock / LPR;  // lane groups (rows) per workgroup
  const int64_t blk = logical_block(blockIdx.x, per_xcd, remap);
  const int64_t r = blk * GPB + threadIdx.x / LPR;
  const int c = (threadIdx.x % LPR) * VEC + blockIdx.y * (LPR * VEC);
  if (r >= n_rows || c >= k) return;
  uint32_t j = rows_ptr[r];
  const uint32_t hi = rows_ptr[r + 1];
  const float* __restrict__ Xc = X + c;
  V acc = vzero<VEC>();
  for (; j + U <= hi; j += U) {
    Entry e[U];
    V x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) e[u] = ent[j + u];
#pragma unroll
    for (int u = 0; u < U; ++u) x[u] = vload<VEC>(Xc + (size_t)e[u].xrow * (size_t)k);
#pragma unroll
    for (int u = 0; u < U; ++u) vfma(acc, e[u].val, x[u]);
  }
  for (; j < hi; ++j) {
    Entry e = ent[j];
    vfma(acc, e.val, vload<VEC>(Xc + (size_t)e.xrow * (size_t)k));
  }
  float* y = Y + (size_t)rows_y[r] * (size_t)k + c;
  if (accumulate) vadd(acc, vload<VEC>(y));
  vstore<VEC>(y, acc);
}

template <int VEC, int LPR, int U>
__global__ __launch_bounds__(kBlock) void chunks_kernel(
    const uint32_t* __restrict__ chunk_ptr, const int32_t* __restrict__ chunk_dst,
    const Entry* __restrict__ ent, int64_t n_chunks, const float* __restrict__ X,
    float* __restrict__ Y, float* __restrict__ partials, int k, int accumulate, int64_t per_xcd,
    int remap) {
  using V = typename Vec<VEC>::type;
  constexpr int G = 64 / LPR;         // lane groups per wavefront
  constexpr int WPB = kBlock / 64;    // wavefronts (chunks) per workgroup
  const int64_t blk = logical_block(blockIdx.x, per_xcd, remap);
  const int64_t ch = blk * WPB + threadIdx.x / 64;
  if (ch >= n_chunks) return;          // whole wavefront leaves together
  const int lane = threadIdx.x % 64;
  const int g = lane / LPR;
  const int c = (lane % LPR) * VEC + blockIdx.y * (LPR * VEC);
  const bool col_ok = c < k;
  const uint32_t lo = chunk_ptr[ch];
  const uint32_t hi = chunk_ptr[ch + 1];
  const float* __restrict__ Xc = X + (col_ok ? c : 0);
  V acc = vzero<VEC>();
  uint32_t j = lo + g;
  // the lane group g takes entries lo+g, lo+g+G, ...
  for (; j + (U - 1) * G < hi; j += U * G) {
    Entry e[U];
    V x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) e[u] = ent[j + u * G];
#pragma unroll
    for (int u = 0; u < U; ++u) x[u] = vload<VEC>(Xc + (size_t)e[u].xrow * (size_t)k);
#pragma unroll
    for (int u = 0; u < U; ++u) vfma(acc, e[u].val, x[u]);
  }
  for (; j < hi; j += G) {
    Entry e = ent[j];
    vfma(acc, e.val, vload<VEC>(Xc + (size_t)e.xrow * (size_t)k));
  }
  // combine the G lane groups: butterfly over lane-id bits LPR, 2 LPR, ..., 32
#pragma unroll
  for (int m = LPR; m < 64; m <<= 1) vadd(acc, vshfl_xor(acc, m));
  if (g == 0 && col_ok) {
    const int32_t dst = chunk_dst[ch];
    if (dst >= 0) {
      float* y = Y + (size_t)dst * (size_t)k + c;
      if (accumulate) vadd(acc, vload<VEC>(y));
      vstore<VEC>(y, acc);
    } else {
      vstore<VEC>(partials + (size_t)(-1 - dst) * (size_t)k + c, acc);
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
  for (uint32_t s = lo + g; s < hi; s += G) vadd(acc, vload<VEC>(Pc + (size_t)s * (size_t)k));
#pragma unroll
  for (int m = LPR; m < 64; m <<= 1) vadd(acc, vshfl_xor(acc, m));
  if (g == 0 && col_ok) {
    float* y = Y + (size_t)split_y[row] * (size_t)k + c;
    if (accumulate) vadd(acc, vload<VEC>(y));
    vstore<VEC>(y, acc);
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

// ---------------------------------------------------------------------------
// host-side dispatch on (VEC, LPR)
// ---------------------------------------------------------------------------
struct Shape {
  int vec, lpr, slices;
};

Shape pick_shape(int k, int kc) {
  Shape s;
  s.vec = (k % 4 == 0) ? 4 : (k % 2 == 0) ? 2 : 1;
  int width = k;                                   // columns per slice
  if (kc > 0 && kc < width) width = kc;
  if (width > 64 * s.vec) width = 64 * s.vec;
  int lanes = (width + s.vec - 1) / s.vec;
  int lpr = 1;
  while (lpr < lanes) lpr <<= 1;
  s.lpr = lpr;
  s.slices = (k + lpr * s.vec - 1) / (lpr * s.vec);
  return s;
}

template <typename F>
int dispatch_shape(const Shape& s, F&& f) {
#define ARROW_CASE(V, L) \
  if (s.vec == V && s.lpr == L) return f(std::integral_constant<int, V>{}, std::integral_constant<int, L>{});
#define ARROW_CASES(V) \
  ARROW_CASE(V, 1) ARROW_CASE(V, 2) ARROW_CASE(V, 4) ARROW_CASE(V, 8) ARROW_CASE(V, 16) ARROW_CASE(V, 32) ARROW_CASE(V, 64)
  ARROW_CASES(4)
  ARROW_CASES(2)
  ARROW_CASES(1)
#undef ARROW_CASES
#undef ARROW_CASE
  return (int)hipErrorInvalidValue;
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace

int launch_rows(const uint32_t* rows_ptr, const int32_t* rows_y, const Entry* entries,
                int64_t n_rows, const float* X, float* Y, int32_t k, bool accumulate,
                const LaunchTuning& t, void* stream) {
  if (n_rows <= 0) return 0;
  const Shape s = pick_shape(k, t.kc);
  return dispatch_shape(s, [&](auto V, auto L) -> int {
    constexpr int VEC = decltype(V)::value, LPR = decltype(L)::value;
    const int64_t blocks = ceil_div(n_rows, kBlock / LPR);
    const int64_t per_xcd = ceil_div(blocks, kXcds);
    const int64_t grid_x = t.xcd_remap ? per_xcd * kXcds : blocks;
    if (grid_x > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)grid_x, (unsigned)s.slices);
    hipLaunchKernelGGL((rows_kernel<VEC, LPR, 4>), grid, dim3(kBlock), 0, (hipStream_t)stream,
                       rows_ptr, rows_y, entries, n_rows, X, Y, (int)k, accumulate ? 1 : 0,
                       per_xcd, t.xcd_remap);
    return (int)hipGetLastError();
  });
}

int launch_chunks(const uint32_t* chunk_ptr, const int32_t* chunk_dst, const Entry* entries,
                  int64_t n_chunks, const float* X, float* Y, float* partials, int32_t k,
                  bool accumulate, const LaunchTuning& t, void* stream) {
  if (n_chunks <= 0) return 0;
  const Shape s = pick_shape(k, t.kc);
  return dispatch_shape(s, [&](auto V, auto L) -> int {
    constexpr int VEC = decltype(V)::value, LPR = decltype(L)::value;
    const int64_t blocks = ceil_div(n_chunks, kBlock / 64);
    const int64_t per_xcd = ceil_div(blocks, kXcds);
    const int64_t grid_x = t.xcd_remap ? per_xcd * kXcds : blocks;
    if (grid_x > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    dim3 grid((unsigned)grid_x, (unsigned)s.slices);
    hipLaunchKernelGGL((chunks_kernel<VEC, LPR, 4>), grid, dim3(kBlock), 0, (hipStream_t)stream,
                       chunk_ptr, chunk_dst, entries, n_chunks, X, Y, partials, (int)k,
                       accumulate ? 1 : 0, per_xcd, t.xcd_remap);
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

}  // namespace arrow
