// Order-3 MTTKRP: host-side compressed-sparse-fibre build and the C boundary.
// The arithmetic of a product happens in the HIP kernels this file launches (mttkrp.hip and the
// shared partial-vector reduction); nothing here falls back to the CPU.
//
// Image: the entries sorted by (i, j, k) as {k, value} pairs; SEGMENTS, runs of at most
// kSegMax entries of one fibre (i, j) with the fibre's j (a long fibre is cut: the product with
// B(j, :) distributes over the pieces); ITEMS, runs of consecutive segments of one slice i with at
// most kItemNnz entries and kItemSegs segments, one per wavefront, with a destination: row i of A when the slice is one
// item, else a partial-vector slot that the reduction pass sums in a fixed order.  Every i in
// [0, I) has at least one item (an empty one stores zeros), so A is fully overwritten.
#include <hip/hip_runtime.h>
#include <omp.h>

#include <algorithm>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "arrow.h"
#include "arrow_internal.h"
#include "csf3.h"

namespace {

thread_local std::string g_err3;

int fail3(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err3 = buf;
  return code;
}

constexpr size_t kAlign3 = 256;
size_t align3(size_t x) { return (x + kAlign3 - 1) / kAlign3 * kAlign3; }
constexpr int64_t kSegMax = arrow::kCsfSegMax;      // most entries of a segment
constexpr int64_t kItemNnz = arrow::kCsfItemNnz;    // an item is closed before it would hold more entries
constexpr int64_t kItemSegs = arrow::kCsfItemSegs;  // ... or more segments than this

}  // namespace

struct csf3_handle {
  int64_t I = 0, J = 0, K = 0, nnz = 0;
  int64_t slices = 0, fibers = 0, n_seg = 0, n_items = 0, n_split = 0, n_partials = 0;
  int64_t distinct_j = 0, distinct_k = 0;
  double build_seconds = 0.0;
  std::vector<unsigned char> bytes;   // packed host copy of the image
  size_t off_seg_ptr = 0, off_seg_j = 0, off_item_seg = 0, off_item_dst = 0, off_item_ent = 0, off_split_ptr = 0,
         off_split_y = 0, off_entries = 0;
  unsigned char* dev = nullptr;
  unsigned char* ws = nullptr;
  size_t ws_bytes = 0;
  bool profiling = false, profiled = false;
  hipEvent_t ev[3] = {nullptr, nullptr, nullptr};   // before the kernel, between, after the reduction
};

extern "C" {

const char* csf3_last_error(void) { return g_err3.c_str(); }

int csf3_build(int64_t I, int64_t J, int64_t K, int64_t nnz, const int32_t* ti, const int32_t* tj,
               const int32_t* tk, const float* tv, csf3_handle** out) {
  if (!out) return fail3(ARROW_EINVAL, "out is NULL");
  *out = nullptr;
  if (I < 1 || J < 1 || K < 1 || I > 2147483647LL || J > 2147483647LL || K > 2147483647LL)
    return fail3(ARROW_EINVAL, "mode sizes must be in [1, 2^31 - 1]");
  if (nnz < 0 || nnz >= 0xffffffffLL) return fail3(ARROW_EINVAL, "nnz must be in [0, 2^32 - 2]");
  if (nnz > 0 && (!ti || !tj || !tk || !tv)) return fail3(ARROW_EINVAL, "a coordinate or value array is NULL");
  auto t0 = std::chrono::steady_clock::now();
  try {
    int64_t bad = -1;
    bool sorted = true;
#pragma omp parallel for schedule(static) reduction(&& : sorted)
    for (int64_t p = 0; p < nnz; ++p) {
      if (ti[p] < 0 || ti[p] >= I || tj[p] < 0 || tj[p] >= J || tk[p] < 0 || tk[p] >= K) {
#pragma omp critical
        if (bad < 0 || p < bad) bad = p;
      }
      if (p > 0) {
        const bool le = ti[p - 1] != ti[p] ? ti[p - 1] < ti[p]
                        : (tj[p - 1] != tj[p] ? tj[p - 1] < tj[p] : tk[p - 1] <= tk[p]);
        sorted = sorted && le;
      }
    }
    if (bad >= 0) return fail3(ARROW_EINVAL, "entry %lld has a coordinate out of range", (long long)bad);
    // order of the entries by (i, j, k); equal coordinates keep the caller's order
    std::vector<uint32_t> order;
    if (!sorted) {
      order.resize((size_t)nnz);
      for (int64_t p = 0; p < nnz; ++p) order[p] = (uint32_t)p;
      std::stable_sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) {
        if (ti[x] != ti[y]) return ti[x] < ti[y];
        if (tj[x] != tj[y]) return tj[x] < tj[y];
        return tk[x] < tk[y];
      });
    }
    auto at = [&](int64_t p) -> int64_t { return sorted ? p : (int64_t)order[p]; };

    csf3_handle* h = new (std::nothrow) csf3_handle;
    if (!h) return fail3(ARROW_ENOMEM, "out of host memory");
    h->I = I; h->J = J; h->K = K; h->nnz = nnz;
    // segments: a new one starts where the fibre changes or the current one is full
    std::vector<uint32_t> seg_ptr;
    std::vector<int32_t> seg_j, seg_i;
    seg_ptr.reserve((size_t)(nnz / 2 + 16));
    for (int64_t p = 0; p < nnz; ++p) {
      const int64_t q = at(p);
      const bool new_fiber = p == 0 || ti[at(p - 1)] != ti[q] || tj[at(p - 1)] != tj[q];
      if (new_fiber) {
        ++h->fibers;
        if (p == 0 || ti[at(p - 1)] != ti[q]) ++h->slices;
      }
      if (new_fiber || (int64_t)(p - seg_ptr.back()) >= kSegMax) {
        seg_ptr.push_back((uint32_t)p);
        seg_j.push_back(tj[q]);
        seg_i.push_back(ti[q]);
      }
    }
    seg_ptr.push_back((uint32_t)nnz);
    h->n_seg = (int64_t)seg_j.size();
    // items: per slice i (empty slices included), consecutive segments up to kItemNnz entries
    // and kItemSegs segments
    std::vector<uint32_t> item_seg, split_ptr;
    std::vector<int32_t> item_dst, split_y;
    split_ptr.push_back(0);
    int64_t s = 0, slots = 0;
    for (int64_t i = 0; i < I; ++i) {
      const size_t first_item = item_dst.size();
      if (s >= h->n_seg || seg_i[s] != i) {          // empty slice: one item without segments
        item_seg.push_back((uint32_t)s);
        item_dst.push_back((int32_t)i);
        continue;
      }
      while (s < h->n_seg && seg_i[s] == i) {
        item_seg.push_back((uint32_t)s);
        item_dst.push_back((int32_t)i);
        int64_t cnt = 0, segs = 0;
        while (s < h->n_seg && seg_i[s] == i && segs < kItemSegs &&
               (cnt == 0 || cnt + (seg_ptr[s + 1] - seg_ptr[s]) <= kItemNnz)) {
          cnt += seg_ptr[s + 1] - seg_ptr[s];
          ++segs;
          ++s;
        }
      }
      const size_t n_it = item_dst.size() - first_item;
      if (n_it > 1) {                                  // split slice: consecutive partial slots
        for (size_t t = 0; t < n_it; ++t) item_dst[first_item + t] = (int32_t)(-1 - (slots + (int64_t)t));
        slots += (int64_t)n_it;
        split_ptr.push_back((uint32_t)slots);
        split_y.push_back((int32_t)i);
      }
    }
    item_seg.push_back((uint32_t)h->n_seg);
    // the kernel stages an item in fixed-size LDS arrays: make sure no item exceeds them
    for (size_t t = 0; t + 1 < item_seg.size(); ++t) {
      const int64_t segs = (int64_t)item_seg[t + 1] - (int64_t)item_seg[t];
      const int64_t ents = (int64_t)seg_ptr[item_seg[t + 1]] - (int64_t)seg_ptr[item_seg[t]];
      if (segs < 0 || segs > kItemSegs || ents < 0 || ents > kItemNnz) {
        delete h;
        return fail3(ARROW_EINTERNAL, "work item %zu holds %lld segments / %lld entries", t, (long long)segs, (long long)ents);
      }
    }
    if (slots > 0x7fffffffLL || item_dst.size() > 0x7fffff00ULL) { delete h; return fail3(ARROW_EINVAL, "too many work items"); }
    h->n_items = (int64_t)item_dst.size();
    h->n_split = (int64_t)split_y.size();
    h->n_partials = slots;
    {
      std::vector<uint8_t> seen_j((size_t)J, 0), seen_k((size_t)K, 0);
      for (int64_t p = 0; p < nnz; ++p) { seen_j[tj[p]] = 1; seen_k[tk[p]] = 1; }
      for (uint8_t v : seen_j) h->distinct_j += v;
      for (uint8_t v : seen_k) h->distinct_k += v;
    }
    size_t total = 0;
    h->off_seg_ptr = total;   total = align3(total + sizeof(uint32_t) * seg_ptr.size());
    h->off_seg_j = total;     total = align3(total + sizeof(int32_t) * seg_j.size());
    h->off_item_seg = total;  total = align3(total + sizeof(uint32_t) * item_seg.size());
    h->off_item_dst = total;  total = align3(total + sizeof(int32_t) * item_dst.size());
    h->off_item_ent = total;  total = align3(total + sizeof(uint32_t) * item_seg.size());
    h->off_split_ptr = total; total = align3(total + sizeof(uint32_t) * split_ptr.size());
    h->off_split_y = total;   total = align3(total + sizeof(int32_t) * split_y.size());
    h->off_entries = total;   total = align3(total + sizeof(arrow::Entry) * (size_t)nnz);
    h->bytes.assign(total, 0);
    unsigned char* base = h->bytes.data();
    std::memcpy(base + h->off_seg_ptr, seg_ptr.data(), sizeof(uint32_t) * seg_ptr.size());
    if (!seg_j.empty()) std::memcpy(base + h->off_seg_j, seg_j.data(), sizeof(int32_t) * seg_j.size());
    std::memcpy(base + h->off_item_seg, item_seg.data(), sizeof(uint32_t) * item_seg.size());
    std::memcpy(base + h->off_item_dst, item_dst.data(), sizeof(int32_t) * item_dst.size());
    {
      uint32_t* item_ent = reinterpret_cast<uint32_t*>(base + h->off_item_ent);
      for (size_t t = 0; t < item_seg.size(); ++t) item_ent[t] = seg_ptr[item_seg[t]];
    }
    std::memcpy(base + h->off_split_ptr, split_ptr.data(), sizeof(uint32_t) * split_ptr.size());
    if (!split_y.empty()) std::memcpy(base + h->off_split_y, split_y.data(), sizeof(int32_t) * split_y.size());
    arrow::Entry* ent = reinterpret_cast<arrow::Entry*>(base + h->off_entries);
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < nnz; ++p) {
      const int64_t q = at(p);
      ent[p].xrow = tk[q];
      ent[p].val = tv[q];
    }
    h->build_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    *out = h;
    return ARROW_OK;
  } catch (const std::bad_alloc&) {
    return fail3(ARROW_ENOMEM, "out of host memory while building the fibre image");
  }
}

size_t csf3_device_bytes(const csf3_handle* h) { return h ? h->bytes.size() : 0; }

int csf3_upload(csf3_handle* h, void* dev_buf, size_t bytes, void* stream) {
  if (!h) return fail3(ARROW_EINVAL, "handle is NULL");
  if (!dev_buf) return fail3(ARROW_EINVAL, "dev_buf is NULL");
  if ((uintptr_t)dev_buf % kAlign3) return fail3(ARROW_EINVAL, "dev_buf must be 256-byte aligned");
  if (bytes < h->bytes.size()) return fail3(ARROW_ETOOSMALL, "image needs %zu bytes, buffer has %zu", h->bytes.size(), bytes);
  if (!h->bytes.empty()) {
    hipError_t e = hipMemcpyAsync(dev_buf, h->bytes.data(), h->bytes.size(), hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e != hipSuccess) return fail3(ARROW_EHIP, "image upload: %s", hipGetErrorString(e));
  }
  h->dev = static_cast<unsigned char*>(dev_buf);
  return ARROW_OK;
}

size_t csf3_workspace_bytes(const csf3_handle* h, int32_t R) {
  if (!h || R < 1) return 0;
  return align3((size_t)h->n_partials * (size_t)R * sizeof(float)) + kAlign3;
}

int csf3_set_workspace(csf3_handle* h, void* dev_ws, size_t bytes) {
  if (!h) return fail3(ARROW_EINVAL, "handle is NULL");
  if (!dev_ws) return fail3(ARROW_EINVAL, "dev_ws is NULL");
  if ((uintptr_t)dev_ws % kAlign3) return fail3(ARROW_EINVAL, "dev_ws must be 256-byte aligned");
  h->ws = static_cast<unsigned char*>(dev_ws);
  h->ws_bytes = bytes;
  return ARROW_OK;
}

int csf3_mttkrp(csf3_handle* h, const float* B, const float* C, float* A, int32_t R, void* stream) {
  if (!h) return fail3(ARROW_EINVAL, "handle is NULL");
  if (R < 1) return fail3(ARROW_EINVAL, "R must be >= 1 (got %d)", R);
  if (!h->dev) return fail3(ARROW_ENOTREADY, "csf3_upload has not been called");
  if (!h->ws) return fail3(ARROW_ENOTREADY, "csf3_set_workspace has not been called");
  if (h->ws_bytes < csf3_workspace_bytes(h, R))
    return fail3(ARROW_ETOOSMALL, "workspace holds %zu bytes, R = %d needs %zu", h->ws_bytes, R, csf3_workspace_bytes(h, R));
  if (!B || !C || !A) return fail3(ARROW_EINVAL, "B, C or A is NULL");
  if (A == B || A == C) return fail3(ARROW_EINVAL, "A must not overlap B or C");
  if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) % 16) return fail3(ARROW_EINVAL, "A, B and C must be 16-byte aligned");
  float* partials = reinterpret_cast<float*>(h->ws);
  auto at = [&](size_t off) { return h->dev + off; };
  const bool prof = h->profiling && h->ev[0];
  if (prof) (void)hipEventRecord(h->ev[0], (hipStream_t)stream);
  int rc = arrow::launch_mttkrp(reinterpret_cast<const uint32_t*>(at(h->off_item_seg)),
                                reinterpret_cast<const uint32_t*>(at(h->off_item_ent)),
                                reinterpret_cast<const int32_t*>(at(h->off_item_dst)),
                                reinterpret_cast<const uint32_t*>(at(h->off_seg_ptr)),
                                reinterpret_cast<const int32_t*>(at(h->off_seg_j)),
                                reinterpret_cast<const arrow::Entry*>(at(h->off_entries)), h->n_items, B,
                                h->J, C, h->K, A, partials, R,
                                h->n_seg ? (double)h->nnz / (double)h->n_seg : 0.0, stream);
  if (rc) return fail3(ARROW_EHIP, "mttkrp kernel launch: %s", hipGetErrorString((hipError_t)rc));
  if (prof) (void)hipEventRecord(h->ev[1], (hipStream_t)stream);
  rc = arrow::launch_reduce(reinterpret_cast<const uint32_t*>(at(h->off_split_ptr)),
                            reinterpret_cast<const int32_t*>(at(h->off_split_y)), h->n_split, partials, A, R,
                            false, stream);
  if (rc) return fail3(ARROW_EHIP, "reduce kernel launch: %s", hipGetErrorString((hipError_t)rc));
  if (prof) { (void)hipEventRecord(h->ev[2], (hipStream_t)stream); h->profiled = true; }
  return ARROW_OK;
}

int csf3_set_profiling(csf3_handle* h, int32_t enabled) {
  if (!h) return fail3(ARROW_EINVAL, "handle is NULL");
  if (enabled && !h->ev[0]) {
    for (hipEvent_t& e : h->ev)
      if (hipEventCreate(&e) != hipSuccess) { e = nullptr; return fail3(ARROW_EHIP, "event creation failed"); }
  }
  h->profiling = enabled != 0;
  h->profiled = false;
  return ARROW_OK;
}

int csf3_get_profile(csf3_handle* h, float* kernel_ms, float* reduce_ms) {
  if (!h || !kernel_ms || !reduce_ms) return fail3(ARROW_EINVAL, "NULL argument");
  if (!h->profiled) return fail3(ARROW_ENOTREADY, "no profiled product has run");
  hipError_t e = hipEventSynchronize(h->ev[2]);
  if (e == hipSuccess) e = hipEventElapsedTime(kernel_ms, h->ev[0], h->ev[1]);
  if (e == hipSuccess) e = hipEventElapsedTime(reduce_ms, h->ev[1], h->ev[2]);
  if (e != hipSuccess) return fail3(ARROW_EHIP, "event timing: %s", hipGetErrorString(e));
  return ARROW_OK;
}

int csf3_info(const csf3_handle* h, csf3_info_t* out) {
  if (!h || !out) return fail3(ARROW_EINVAL, "NULL argument");
  out->I = h->I; out->J = h->J; out->K = h->K; out->nnz = h->nnz;
  out->slices = h->slices; out->fibers = h->fibers; out->segments = h->n_seg; out->items = h->n_items;
  out->split_rows = h->n_split; out->partials = h->n_partials;
  out->distinct_j = h->distinct_j; out->distinct_k = h->distinct_k;
  out->build_seconds = h->build_seconds;
  return ARROW_OK;
}

void csf3_destroy(csf3_handle* h) {
  if (!h) return;
  for (hipEvent_t e : h->ev)
    if (e) (void)hipEventDestroy(e);
  delete h;
}

}  // extern "C"
