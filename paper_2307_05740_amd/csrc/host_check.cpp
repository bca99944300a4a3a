// Host-only exerciser of everything in the library that runs on the CPU, meant to be built with
// -fsanitize=address,undefined (see _build.build_host_check): validation of the caller's CSR, the
// arrow decomposition, the image packer under many option sets, the image self-check, export,
// save / load / repack, and the compressed-sparse-fibre builder of the order-3 MTTKRP.  No GPU is
// involved and no kernel runs: the kernel launchers and the few HIP runtime calls the boundary
// makes are replaced by stubs below that fail loudly if anything reaches them.
// Exit status 0 = every step did what it should (and the sanitizers had nothing to report).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "arrow.h"
#include "arrow_internal.h"
#include "csf3.h"

// ---- stubs: nothing below may be reached by a host-only run ---------------------------------------
[[noreturn]] static void reached(const char* what) {
  std::fprintf(stderr, "host_check: %s was called in a host-only run\n", what);
  std::abort();
}
extern "C" {
const char* hipGetErrorString(hipError_t) { return "host-only build"; }
hipError_t hipEventCreate(hipEvent_t*) { reached("hipEventCreate"); }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { reached("hipEventRecord"); }
hipError_t hipEventSynchronize(hipEvent_t) { reached("hipEventSynchronize"); }
hipError_t hipEventElapsedTime(float*, hipEvent_t, hipEvent_t) { reached("hipEventElapsedTime"); }
hipError_t hipEventDestroy(hipEvent_t) { reached("hipEventDestroy"); }
hipError_t hipMemcpyAsync(void*, const void*, size_t, hipMemcpyKind, hipStream_t) { reached("hipMemcpyAsync"); }
}
namespace arrow {
int launch_rows(const uint32_t*, const uint32_t*, const int32_t*, const Entry*, int64_t, const float*, int64_t,
                const float*, float*, float*, int32_t, bool, const LaunchTuning&, void*) { reached("launch_rows"); }
int launch_chunks(const uint32_t*, const uint32_t*, const int32_t*, const Entry*, int64_t, const float*, int64_t,
                  const float*, float*, float*, int32_t, bool, const LaunchTuning&, void*) { reached("launch_chunks"); }
int launch_reduce(const uint32_t*, const int32_t*, int64_t, const float*, float*, int32_t, bool, void*) { reached("launch_reduce"); }
int launch_gather(const int32_t*, int64_t, const float*, float*, int32_t, void*) { reached("launch_gather"); }
int launch_panel(const uint32_t*, const int32_t*, const Entry*, int64_t, const float*, int64_t, float*, int32_t, void*) { reached("launch_panel"); }
int launch_panel_combine(const int32_t*, int64_t, const float*, float*, int32_t, void*) { reached("launch_panel_combine"); }
int launch_sddmm_panel(const uint32_t*, const int32_t*, const Entry*, const uint32_t*, int64_t, const float*,
                       const float*, int64_t, float*, int32_t, void*) { reached("launch_sddmm_panel"); }
int launch_corner(const uint32_t*, const uint32_t*, int64_t, const Entry*, const float*, int64_t, float*, int32_t, void*) { reached("launch_corner"); }
int launch_corner_combine(const uint32_t*, const int32_t*, int64_t, const float*, float*, int32_t, void*) { reached("launch_corner_combine"); }
int launch_sddmm_corner(const uint32_t*, int64_t, const int32_t*, const Entry*, const uint32_t*, const float*,
                        const float*, int64_t, float*, int32_t, void*) { reached("launch_sddmm_corner"); }
int launch_window(const WindowTile*, int64_t, int64_t, const uint32_t*, const uint32_t*, const int32_t*, const Entry*,
                  const int32_t*, const float*, float*, int32_t, bool, void*) { reached("launch_window"); }
int launch_sddmm_rows(int, const uint32_t*, const uint32_t*, const int32_t*, const uint32_t*, const int32_t*,
                      const Entry*, const uint32_t*, int64_t, const float*, const float*, int64_t, const float*,
                      float*, int32_t, void*) { reached("launch_sddmm_rows"); }
int launch_sddmm_chunks(const uint32_t*, const uint32_t*, const int32_t*, const Entry*, const uint32_t*, int64_t,
                        const float*, const float*, int64_t, const float*, float*, int32_t, void*) { reached("launch_sddmm_chunks"); }
unsigned char* static_scratch(std::string&) { reached("static_scratch"); }
int64_t probe_out_floats(int64_t) { reached("probe_out_floats"); }
int launch_probe_gather(const float*, int64_t, int32_t, int64_t, int, int, int64_t, float*, void*) { reached("launch_probe_gather"); }
int launch_mttkrp(const uint32_t*, const uint32_t*, const int32_t*, const uint32_t*, const int32_t*, const Entry*,
                  int64_t, const float*, int64_t, const float*, int64_t, float*, float*, int32_t, double, void*) { reached("launch_mttkrp"); }
}  // namespace arrow

// ---- operands ---------------------------------------------------------------------------------------
namespace {

struct Csr {
  int64_t n = 0;
  std::vector<int64_t> rowptr;
  std::vector<int32_t> col;
  std::vector<float> val;
};

uint64_t next_u64(uint64_t& s) {          // xorshift64*
  s ^= s >> 12; s ^= s << 25; s ^= s >> 27;
  return s * 0x2545F4914F6CDD1DULL;
}

Csr from_pairs(int64_t n, std::vector<std::pair<int32_t, int32_t>> e, uint64_t seed) {
  std::sort(e.begin(), e.end());
  e.erase(std::unique(e.begin(), e.end()), e.end());
  Csr a;
  a.n = n;
  a.rowptr.assign(n + 1, 0);
  for (auto& p : e) ++a.rowptr[p.first + 1];
  for (int64_t i = 0; i < n; ++i) a.rowptr[i + 1] += a.rowptr[i];
  for (auto& p : e) {
    a.col.push_back(p.second);
    a.val.push_back((float)((double)(next_u64(seed) >> 40) / (double)(1 << 23) - 1.0));
  }
  return a;
}

// skewed graph: both endpoints drawn with a quadrant recursion that prefers low ids
Csr skewed(int scale, int64_t samples, bool symmetric, uint64_t seed) {
  const int64_t n = 1LL << scale;
  std::vector<std::pair<int32_t, int32_t>> e;
  for (int64_t s = 0; s < samples; ++s) {
    int32_t u = 0, v = 0;
    for (int b = 0; b < scale; ++b) {
      const uint64_t r = next_u64(seed) % 100;
      const int q = r < 57 ? 0 : (r < 76 ? 1 : (r < 95 ? 2 : 3));
      u = (u << 1) | (q >> 1);
      v = (v << 1) | (q & 1);
    }
    e.emplace_back(u, v);
    if (symmetric) e.emplace_back(v, u);
  }
  return from_pairs(n, std::move(e), seed + 1);
}

Csr grid(int N) {
  std::vector<std::pair<int32_t, int32_t>> e;
  for (int y = 0; y < N; ++y)
    for (int x = 0; x < N; ++x) {
      const int32_t v = y * N + x;
      e.emplace_back(v, v);
      if (x) e.emplace_back(v, v - 1);
      if (x + 1 < N) e.emplace_back(v, v + 1);
      if (y) e.emplace_back(v, v - N);
      if (y + 1 < N) e.emplace_back(v, v + N);
    }
  return from_pairs((int64_t)N * N, std::move(e), 7);
}

Csr shift(int64_t n, int64_t off, int64_t cnt) {
  std::vector<std::pair<int32_t, int32_t>> e;
  for (int64_t i = 0; i < cnt; ++i) e.emplace_back((int32_t)i, (int32_t)(i + off));
  return from_pairs(n, std::move(e), 9);
}

int failures = 0;
#define EXPECT(cond, ...)                                              \
  do {                                                                 \
    if (!(cond)) {                                                     \
      std::fprintf(stderr, "host_check: FAILED %s: ", #cond);          \
      std::fprintf(stderr, __VA_ARGS__);                               \
      std::fprintf(stderr, " (%s)\n", arrow_last_error());             \
      ++failures;                                                      \
    }                                                                  \
  } while (0)

// every level's entries, mapped back, counted per (row, col): must be A's pattern exactly once
void check_levels(const Csr& a, arrow_handle* h, const char* what) {
  arrow_info_t info;
  EXPECT(arrow_info(h, &info) == ARROW_OK && info.n == a.n && info.nnz == a.rowptr[a.n], "%s: info", what);
  std::vector<uint8_t> seen(a.col.size(), 0);
  for (int32_t li = 0; li < info.levels; ++li) {
    arrow_level_info_t L;
    EXPECT(arrow_level_info(h, li, &L) == ARROW_OK, "%s: level info", what);
    std::vector<int32_t> perm(L.n_i), r(L.nnz), c(L.nnz);
    std::vector<float> v(L.nnz);
    EXPECT(arrow_export_level(h, li, perm.data(), r.data(), c.data(), v.data()) == ARROW_OK, "%s: export", what);
    for (int64_t e = 0; e < L.nnz; ++e) {
      const int64_t p = r[e], q = c[e];
      EXPECT(p < info.b || q < info.b || p / info.b == q / info.b, "%s: entry outside the arrow", what);
      const int32_t u = perm[p], w = perm[q];
      const int32_t* cb = a.col.data() + a.rowptr[u];
      const int32_t* ce = a.col.data() + a.rowptr[u + 1];
      const int32_t* it = std::lower_bound(cb, ce, w);
      const bool found = it != ce && *it == w;
      EXPECT(found, "%s: a level entry is not in A", what);
      if (!found) return;
      const size_t at = (size_t)(it - a.col.data());
      EXPECT(!seen[at] && std::memcmp(&a.val[at], &v[e], 4) == 0, "%s: entry repeated or value changed", what);
      seen[at] = 1;
    }
  }
  EXPECT(std::count(seen.begin(), seen.end(), 1) == (int64_t)seen.size(), "%s: entries missing", what);
}

void run_operand(const Csr& a, int32_t b, const char* name, const std::string& tmp) {
  struct Variant { const char* what; void (*set)(arrow_options_t&); };
  const Variant variants[] = {
      {"defaults", [](arrow_options_t&) {}},
      {"levels not fused, tiny chunks", [](arrow_options_t& o) { o.fuse_levels = 0; o.chunk_nnz = 7; o.short_max = 3; o.window_rows = 64; }},
      {"dense corner", [](arrow_options_t& o) { o.corner = 1; o.hubs_first = 65536; o.corner_min_tile = 1; }},
      {"head panels", [](arrow_options_t& o) { o.panel = 1; o.window_rows = 32; o.panel_min = 1; o.short_max = 0; }},
      {"die queues", [](arrow_options_t& o) { o.classes = 16; o.class_min = 2; o.class_gran = 16; o.piece_max = 5; }},
      {"no separators, id order, LDS windows", [](arrow_options_t& o) { o.separators = 0; o.bfs_tail = 0; o.window_reuse = 0.5; o.window_level_share = 0.0; o.stage_head = 0; }},
  };
  for (const Variant& var : variants) {
    arrow_options_t opt;
    arrow_options_default(&opt);
    var.set(opt);
    arrow_handle* h = nullptr;
    int rc = arrow_decompose_with(a.n, a.rowptr.data(), a.col.data(), a.val.data(), b, &opt, &h);
    EXPECT(rc == ARROW_OK && h, "%s / %s: decompose", name, var.what);
    if (!h) continue;
    EXPECT(arrow_self_check(h) == ARROW_OK, "%s / %s: self check", name, var.what);
    check_levels(a, h, name);
    EXPECT(arrow_device_bytes(h) > 0 && arrow_workspace_bytes(h, 20) >= (size_t)a.n * 80, "%s: sizes", name);
    std::vector<uint32_t> emap((size_t)a.rowptr[a.n]);
    EXPECT(arrow_export_entry_map(h, emap.data()) == ARROW_OK, "%s: entry map", name);
    // compute calls without an uploaded image are refused before anything is launched
    EXPECT(arrow_spmm(h, (const float*)16, (float*)4096, 4, nullptr) == ARROW_ENOTREADY, "%s: spmm before upload", name);
    EXPECT(arrow_spmm_static(h, (const float*)16, (float*)4096, 4, nullptr) == ARROW_ENOTREADY, "%s: static before upload", name);
    // save, load with other options, repack
    EXPECT(arrow_save(h, tmp.c_str()) == ARROW_OK, "%s / %s: save", name, var.what);
    arrow_options_t other;
    arrow_options_default(&other);
    other.chunk_nnz = 33;
    arrow_handle* g = nullptr;
    EXPECT(arrow_load_with(tmp.c_str(), &other, &g) == ARROW_OK && g, "%s / %s: load", name, var.what);
    if (g) {
      EXPECT(arrow_self_check(g) == ARROW_OK, "%s / %s: self check of the loaded handle", name, var.what);
      check_levels(a, g, name);
      EXPECT(arrow_repack(g, &opt) == ARROW_OK && arrow_self_check(g) == ARROW_OK, "%s / %s: repack", name, var.what);
      arrow_destroy(g);
    }
    arrow_destroy(h);
  }
}

}  // namespace

int main(int argc, char** argv) {
  const std::string tmp = argc > 1 ? argv[1] : "/tmp/arrow_host_check.levels";
  run_operand(skewed(12, 40000, true, 1), 256, "skewed symmetric", tmp);
  run_operand(skewed(11, 30000, false, 2), 100, "skewed directed", tmp);
  run_operand(grid(48), 512, "grid", tmp);
  run_operand(shift(4096, 100, 3796), 64, "directed shift", tmp);
  run_operand(shift(64, 32, 28), 4, "small directed shift", tmp);
  {
    // malformed operands and arguments
    Csr a = grid(8);
    arrow_handle* h = nullptr;
    std::vector<int32_t> bad = a.col;
    bad[3] = (int32_t)a.n;
    EXPECT(arrow_decompose(a.n, a.rowptr.data(), bad.data(), a.val.data(), 4, &h) == ARROW_EINVAL && !h, "column out of range");
    bad = a.col;
    std::swap(bad[0], bad[1]);
    EXPECT(arrow_decompose(a.n, a.rowptr.data(), bad.data(), a.val.data(), 4, &h) == ARROW_EINVAL && !h, "unsorted row");
    EXPECT(arrow_decompose(a.n, a.rowptr.data(), a.col.data(), a.val.data(), 0, &h) == ARROW_EINVAL, "b = 0");
    EXPECT(arrow_decompose(0, a.rowptr.data(), a.col.data(), a.val.data(), 4, &h) == ARROW_EINVAL, "n = 0");
    EXPECT(arrow_load("/nonexistent/arrow.levels", &h) == ARROW_EINVAL && !h, "load of a missing file");
    // a truncated file is refused
    EXPECT(arrow_decompose(a.n, a.rowptr.data(), a.col.data(), a.val.data(), 4, &h) == ARROW_OK, "grid 8");
    if (h) {
      EXPECT(arrow_save(h, tmp.c_str()) == ARROW_OK, "save");
      arrow_destroy(h);
      h = nullptr;
      std::FILE* f = std::fopen(tmp.c_str(), "rb");
      std::vector<char> blob;
      if (f) { char buf[4096]; size_t got; while ((got = std::fread(buf, 1, sizeof buf, f)) > 0) blob.insert(blob.end(), buf, buf + got); std::fclose(f); }
      f = std::fopen(tmp.c_str(), "wb");
      if (f) { std::fwrite(blob.data(), 1, blob.size() / 2, f); std::fclose(f); }
      EXPECT(arrow_load(tmp.c_str(), &h) == ARROW_EINVAL && !h, "truncated file");
    }
    arrow_destroy(nullptr);
  }
  {
    // order-3 tensor: 40^3 cube, 3000 entries with duplicates
    uint64_t s = 5;
    std::vector<int32_t> ti, tj, tk;
    std::vector<float> tv;
    for (int e = 0; e < 3000; ++e) {
      ti.push_back((int32_t)(next_u64(s) % 40)); tj.push_back((int32_t)(next_u64(s) % 40));
      tk.push_back((int32_t)(next_u64(s) % 7)); tv.push_back((float)(e % 13) - 6.f);
    }
    csf3_handle* t = nullptr;
    EXPECT(csf3_build(40, 40, 7, (int64_t)tv.size(), ti.data(), tj.data(), tk.data(), tv.data(), &t) == 0 && t, "csf3_build");
    if (t) {
      csf3_info_t ci;
      EXPECT(csf3_info(t, &ci) == 0 && ci.nnz == 3000 && ci.I == 40, "csf3_info");
      EXPECT(csf3_device_bytes(t) > 0 && csf3_workspace_bytes(t, 16) > 0, "csf3 sizes");
      csf3_destroy(t);
    }
    tk[5] = 7;
    EXPECT(csf3_build(40, 40, 7, (int64_t)tv.size(), ti.data(), tj.data(), tk.data(), tv.data(), &t) != 0, "csf3 index out of range");
  }
  std::remove(tmp.c_str());
  if (failures) { std::fprintf(stderr, "host_check: %d failure(s)\n", failures); return 1; }
  std::printf("host_check: ok\n");
  return 0;
}
