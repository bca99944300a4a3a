// Helpers shared by the HIP kernel files: vector types over VEC columns, row loads, the
// wavefront-private LDS strip barrier, and the host-side choice of the (VEC, LPR) shape.
// Everything has internal linkage; include inside a .hip file only.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "arrow_internal.h"

namespace arrow {
namespace {

constexpr int kBlock = 64 * kChunksPerGroup;  // threads per workgroup = 4 wavefronts

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

// Store of a result row that this product does not read again: the non-temporal hint keeps the
// 4 k bytes per output row from displacing rows of X in the L2 (measured on the R-MAT workload:
// rows kernel 3.97 -> 3.71 ms, reduction 0.38 -> 0.33 ms; the same hint on loads of X rows or of
// the entry stream made the product slower).
typedef float stream_v2f __attribute__((ext_vector_type(2)));
typedef float stream_v4f __attribute__((ext_vector_type(4)));
template <int VEC>
__device__ __forceinline__ void vstore_stream(float* p, typename Vec<VEC>::type v);
template <> __device__ __forceinline__ void vstore_stream<1>(float* p, float v) { __builtin_nontemporal_store(v, p); }
template <> __device__ __forceinline__ void vstore_stream<2>(float* p, float2 v) {
  stream_v2f t; t.x = v.x; t.y = v.y;
  __builtin_nontemporal_store(t, reinterpret_cast<stream_v2f*>(p));
}
template <> __device__ __forceinline__ void vstore_stream<4>(float* p, float4 v) {
  stream_v4f t; t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
  __builtin_nontemporal_store(t, reinterpret_cast<stream_v4f*>(p));
}

// Load of a row that is read exactly once (a partial vector in the reduction, the old value of a
// Y row a later level adds to), same hint.
template <int VEC>
__device__ __forceinline__ typename Vec<VEC>::type vload_stream(const float* p);
template <> __device__ __forceinline__ float vload_stream<1>(const float* p) { return __builtin_nontemporal_load(p); }
template <> __device__ __forceinline__ float2 vload_stream<2>(const float* p) {
  stream_v2f t = __builtin_nontemporal_load(reinterpret_cast<const stream_v2f*>(p)); return make_float2(t.x, t.y);
}
template <> __device__ __forceinline__ float4 vload_stream<4>(const float* p) {
  stream_v4f t = __builtin_nontemporal_load(reinterpret_cast<const stream_v4f*>(p)); return make_float4(t.x, t.y, t.z, t.w);
}

// Load VEC columns of row `row` of a row-major matrix.  `base` is wavefront-uniform,
// col_bytes the lane's byte offset inside a row, row_bytes = 4 k.
// SMALL: the matrix has at most 2^24 rows and 2^32 bytes, so the byte offset is one 24-bit
// multiply-add and the load can use (uniform base + 32-bit lane offset) addressing.
template <int VEC, bool SMALL>
__device__ __forceinline__ typename Vec<VEC>::type load_row(const char* base, int32_t row,
                                                            uint32_t row_bytes, uint32_t col_bytes) {
  if (SMALL) {
    const uint32_t off = __umul24((uint32_t)row, row_bytes) + col_bytes;
    return *reinterpret_cast<const typename Vec<VEC>::type*>(base + off);
  } else {
    const uint64_t off = (uint64_t)(uint32_t)row * row_bytes + col_bytes;
    return *reinterpret_cast<const typename Vec<VEC>::type*>(base + off);
  }
}

__device__ __forceinline__ void strip_sync() {
  // the strip is written and read by lanes of ONE wavefront: LDS executes a wavefront's
  // instructions in order, so only the compiler has to be kept from reordering
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---------------------------------------------------------------------------
// host-side dispatch on (VEC, LPR)
// ---------------------------------------------------------------------------
struct Shape {
  int vec, lpr, slices;
};

[[maybe_unused]] Shape pick_shape(int k, int kc) {
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

// 32-bit offsets are enough when a matrix of `rows` rows and k columns stays below 2^24 rows
// and 2^32 bytes (and a row below 2^24 bytes, for the 24-bit multiply)
inline bool small_matrix(int64_t rows, int32_t k) {
  return rows <= (1LL << 24) && rows * (int64_t)k * 4 <= (1LL << 32) && (int64_t)k * 4 < (1LL << 24);
}

}  // namespace
}  // namespace arrow
