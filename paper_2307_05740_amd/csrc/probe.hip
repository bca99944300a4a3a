// Measurement aid, not part of the product: a bare row gather, the yardstick the product's
// kernels are compared with.  Every lane group of 4 k / 16 lanes reads whole rows of a row-major
// fp32 matrix (one 16-byte load per lane, eight rows in flight per lane group) at pseudo-random
// row numbers drawn from a region of the matrix, and adds them up; nothing else happens, so the
// rate is what the memory level that holds the region can deliver to this access pattern:
//   region_rows * 4k bytes <= ~2 MiB, per_die = 1 : every accelerator die draws from its own
//                                         region, which stays in the die's L2 (L2 hits)
//   region of 128 MiB, per_die = 0          : the size of the staged head of the headline workload
//   the whole matrix (GiBs)                 : HBM
//   from_lds = 1                            : the region (at most 64 KiB) is copied into LDS first
// The row numbers come from a hash of the gather's index, so a run is repeatable.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "arrow_internal.h"
#include "kernel_common.h"

namespace arrow {
namespace {

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du;
  x ^= x >> 15; x *= 0x846ca68bu;
  x ^= x >> 16;
  return x;
}

constexpr int kProbeU = 8;             // rows in flight per lane group
constexpr int kProbePerWave = 2048;    // gathers a wavefront performs ...
constexpr int kProbeLdsReps = 16;      // ... times this when the region is read from LDS (the copy into LDS is paid once)

// k % 4 == 0, k <= 256: LPR = k / 4 lanes cover a row, G = 64 / LPR lane groups per wavefront
template <int LPR, bool LDS>
__global__ __launch_bounds__(kBlock) void probe_gather_kernel(const float* __restrict__ X, uint32_t region_rows,
                                                              int per_die, int k, float* __restrict__ out) {
  constexpr int G = 64 / LPR;
  extern __shared__ float win[];
  const int lane = threadIdx.x % 64;
  const int g = lane / LPR;
  const int l = lane % LPR;
  const uint32_t wave_id = blockIdx.x * (kBlock / 64) + threadIdx.x / 64;
  const uint32_t die = blockIdx.x % kDies;                      // workgroups go to the dies round-robin
  const size_t base_row = per_die ? (size_t)die * region_rows : 0;
  const uint32_t row_bytes = 4u * (uint32_t)k;
  if (LDS) {
    for (uint32_t i = threadIdx.x; i < region_rows * (uint32_t)LPR; i += kBlock)
      vstore<4>(win + (size_t)i * 4, vload<4>(X + (base_row + i / LPR) * (size_t)k + (i % LPR) * 4));
    __syncthreads();
  }
  const char* base = reinterpret_cast<const char*>(LDS ? win : X + base_row * (size_t)k);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  const bool pow2 = (region_rows & (region_rows - 1)) == 0;
  for (uint32_t s = 0; s < (LDS ? kProbeLdsReps : 1) * (kProbePerWave / G); s += kProbeU) {
    uint32_t row[kProbeU];
    float4 x[kProbeU];
#pragma unroll
    for (int u = 0; u < kProbeU; ++u)
    {
      // a power-of-two region (every region bench.py uses) needs a mask, not a division: with the
      // rows in LDS the division would be what the probe measures
      const uint32_t idx = wave_id * (LDS ? kProbeLdsReps : 1) * kProbePerWave + (s + u) * G + g;
      // a multiplicative hash (one multiply, one shift) where a mask selects the row; the full
      // mixing function only where a division is needed anyway
      row[u] = pow2 ? (((idx * 0x9E3779B1u) >> 9) & (region_rows - 1)) : (mix32(idx) % region_rows);
    }
#pragma unroll
    for (int u = 0; u < kProbeU; ++u)
      x[u] = *reinterpret_cast<const float4*>(base + (size_t)row[u] * row_bytes + 16u * l);
#pragma unroll
    for (int u = 0; u < kProbeU; ++u) { acc.x += x[u].x; acc.y += x[u].y; acc.z += x[u].z; acc.w += x[u].w; }
  }
  out[(size_t)wave_id * 64 + lane] = acc.x + acc.y + acc.z + acc.w;
}

}  // namespace

// gathers = rows read in total (rounded up to whole wavefronts of kProbePerWave); `out` needs
// 64 floats per wavefront: probe_out_floats(gathers)
int64_t probe_out_floats(int64_t gathers) {
  return ceil_div(ceil_div(gathers, kProbePerWave), kBlock / 64) * (kBlock / 64) * 64;
}

int launch_probe_gather(const float* X, int64_t x_rows, int32_t k, int64_t region_rows, int per_die,
                        int from_lds, int64_t gathers, float* out, void* stream) {
  if (k < 4 || k > 256 || k % 4 || (k & (k - 1))) return (int)hipErrorInvalidValue;   // 4, 8, ..., 256
  if (region_rows < 1 || region_rows > 0xffffffffLL || gathers < 1) return (int)hipErrorInvalidValue;
  if ((per_die ? region_rows * kDies : region_rows) > x_rows) return (int)hipErrorInvalidValue;
  const int64_t lds_bytes = from_lds ? region_rows * (int64_t)k * 4 : 0;
  if (lds_bytes > 64 * 1024) return (int)hipErrorInvalidValue;
  const int64_t blocks = ceil_div(ceil_div(gathers, kProbePerWave * (from_lds ? kProbeLdsReps : 1)), kBlock / 64);
  if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
  const int lpr = k / 4;
#define ARROW_PROBE(L)                                                                                  \
  if (lpr == L) {                                                                                       \
    if (from_lds)                                                                                       \
      hipLaunchKernelGGL((probe_gather_kernel<L, true>), dim3((unsigned)blocks), dim3(kBlock), (size_t)lds_bytes, \
                         (hipStream_t)stream, X, (uint32_t)region_rows, per_die, (int)k, out);         \
    else                                                                                                \
      hipLaunchKernelGGL((probe_gather_kernel<L, false>), dim3((unsigned)blocks), dim3(kBlock), 0,      \
                         (hipStream_t)stream, X, (uint32_t)region_rows, per_die, (int)k, out);         \
    return (int)hipGetLastError();                                                                      \
  }
  ARROW_PROBE(1) ARROW_PROBE(2) ARROW_PROBE(4) ARROW_PROBE(8) ARROW_PROBE(16) ARROW_PROBE(32) ARROW_PROBE(64)
#undef ARROW_PROBE
  return (int)hipErrorInvalidValue;
}

}  // namespace arrow
